// C-ABI layer of libtng: argument checking, workspace partition, and the call sequence of one
// TNG iteration (Algorithm 1 of arXiv 1901.08227 with the normalisation of Eqs. 1-2).
#include "../../include/tng.h"

#include "tng_device.hpp"
#include "tng_kernels.hpp"

#include <cmath>
#include <mutex>
#include <new>
#include <vector>

struct tng_ctx {
  tng_config cfg;
  hipStream_t stream;
  tng::CodecShape shape;
  // workspace partition (device)
  uint32_t* idx;          // [M][batch] minibatch row ids
  float* resid;           // [M][batch] sigma(z) - y
  const void** tables;    // 6 tables of M entries: X|rowptr, col, val, y, n_rows, per-row tile index (CSR)
  std::vector<uint64_t> n_rows;  // host copy of the row counts
  bool have_index;        // the CSR tile index has been built for the current shards
  float* partials;        // [kAbsmaxMaxBlocks][M] partial maxima of the scale pass
  int64_t* rowbase;       // [M][batch] start of each minibatch row in the worker's CSR arrays
  uint32_t* bounds;       // [M][tiles+1][batch] segment bounds of the CSR gradient
  float* zpart;           // [M][tiles][batch] per-tile partial dot products of the CSR gradient
  bool have_dense, have_csr;
  bool csr_pairs;         // the CSR shards hold (column, value) pairs instead of two arrays
  const float* noise;     // Rosenbrock noise, may be null
  float noise_sigma;      // > 0: Gaussian noise is generated on the device instead
  const float* gref2;     // second reference of the combined normalisation
  float* history;         // [ref_window][d] ring of decoded averages (window-average reference)
  float* parts;           // dense problem, wide rows: partial gradients [M][splits][d] of the one-pass kernel, or null
  uint32_t* check;        // CSR problem: flag word of tng_validate_csr, then uint64[M] entry counts at +256 bytes
  double* sums;           // chunk and group sums of the order-pinned row sums (mean reference, l2 scale)
  void* cand;             // scratch of the ternary coder that reads g once (candidate slots), or null
  std::vector<hipEvent_t> prof;  // optional timing events, 5 per slot
  uint32_t prof_slots;
  uint64_t enc_calls, dec_calls;
};

// Scratch of tng_normalize_encode_static: the partial maxima of the scale pass for up to
// kStaticMaxWorkers workers, resident on every GPU the library runs on until the process ends.  In host
// code this name is only a handle for hipGetSymbolAddress; kernels get the address that call returns.
constexpr uint32_t kStaticMaxWorkers = 64;
constexpr size_t kStaticScratchBytes = (size_t)tng::kAbsmaxMaxBlocks * kStaticMaxWorkers * sizeof(float);  // 1 MiB
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr size_t kAlign = 256;
inline size_t round_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }
inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

bool config_valid(const tng_config* c) {
  if (c == nullptr) return false;
  if (c->d == 0 || c->d > (1ull << 34)) return false;
  if (c->M == 0 || c->M > 65535u) return false;
  if (c->bits != 2 && c->bits != 4) return false;
  if (c->norm < TNG_NORM_NONE || c->norm > TNG_NORM_MEAN) return false;
  if (c->scale != TNG_SCALE_MAX && c->scale != TNG_SCALE_L2) return false;
  if (!(c->quot_eps > 0.0f) || !std::isfinite(c->quot_eps)) return false;
  if (c->ref_policy < TNG_REF_ZERO || c->ref_policy > TNG_REF_WINDOW_AVG) return false;
  if (c->ref_policy == TNG_REF_WINDOW_AVG && (c->ref_window == 0 || c->ref_window > 65536u)) return false;
  if (c->ref_period == 0) return false;
  if (!std::isfinite(c->lr) || !std::isfinite(c->l2)) return false;
  if (c->problem < TNG_PROB_EXTERNAL || c->problem > TNG_PROB_ROSENBROCK) return false;
  const bool logreg = c->problem == TNG_PROB_LOGREG_DENSE || c->problem == TNG_PROB_LOGREG_CSR;
  if (logreg && c->batch == 0) return false;
  // CSR columns are int32 and the column tiles of its kernels are one grid dimension (at most 65535)
  if (c->problem == TNG_PROB_LOGREG_CSR && c->d > (65535ull << tng::kCsrTileShift)) return false;
  return true;
}

tng::CodecShape shape_of(const tng_config* cfg) {
  tng::CodecShape sh{};
  const uint64_t per = 32 / cfg->bits;
  sh.d = cfg->d;
  sh.words = (cfg->d + per - 1) / per;
  sh.M = cfg->M;
  sh.bits = (int)cfg->bits;
  sh.norm = cfg->norm;
  sh.eps = cfg->quot_eps;
  sh.k0 = (uint32_t)(cfg->seed & 0xFFFFFFFFull);
  sh.k1 = (uint32_t)(cfg->seed >> 32);
  sh.scale_l2 = cfg->scale == TNG_SCALE_L2 ? 1 : 0;
  sh.means = nullptr;
  return sh;
}

struct Partition {
  size_t idx_off, resid_off, tables_off, partials_off, rowbase_off, bounds_off, zpart_off, sums_off, check_off, parts_off,
      cand_off, cand_bytes, total;
};

Partition partition(const tng_config* c) {
  Partition p{};
  const bool logreg = c->problem == TNG_PROB_LOGREG_DENSE || c->problem == TNG_PROB_LOGREG_CSR;
  const size_t mb = logreg ? (size_t)c->M * c->batch : 0;
  size_t off = 0;
  p.idx_off = off;
  off += round_up(mb * sizeof(uint32_t));
  p.resid_off = off;
  off += round_up(mb * sizeof(float));
  p.tables_off = off;
  off += round_up(logreg ? (size_t)c->M * 6 * sizeof(void*) : 0);
  p.partials_off = off;
  off += round_up((size_t)tng::kAbsmaxMaxBlocks * c->M * sizeof(float));
  p.rowbase_off = off;
  if (c->problem == TNG_PROB_LOGREG_CSR) off += round_up((size_t)c->M * c->batch * sizeof(int64_t));
  p.bounds_off = off;
  if (c->problem == TNG_PROB_LOGREG_CSR)
    off += round_up((size_t)c->M * c->batch * (tng::csr_tiles(c->d) + 1) * sizeof(uint32_t));
  p.zpart_off = off;
  if (c->problem == TNG_PROB_LOGREG_CSR)
    off += round_up((size_t)c->M * c->batch * tng::csr_tiles(c->d) * sizeof(float));
  p.sums_off = off;
  if (c->norm == TNG_NORM_MEAN || c->scale == TNG_SCALE_L2)
    off += round_up(tng::tree_sum_scratch(c->d, c->M) * sizeof(double));
  p.check_off = off;  // tng_validate_csr: a flag word and the per-worker entry counts
  if (c->problem == TNG_PROB_LOGREG_CSR) off += round_up(256 + (size_t)c->M * sizeof(uint64_t));
  p.parts_off = off;  // dense problem, wide rows: per-workgroup partial gradients of the one-pass kernel
  if (c->problem == TNG_PROB_LOGREG_DENSE)
    off += round_up((size_t)tng::dense_row_splits(c->d, c->M, c->batch) * c->M * c->d * sizeof(float));
  p.cand_off = off;  // ternary coder that reads g once: sample maxima and candidate slots
  p.cand_bytes = tng::candidate_scratch_bytes(shape_of(c));
  off += round_up(p.cand_bytes);
  p.total = off;
  return p;
}

inline bool refresh_now(const tng_config& c, uint32_t iter) {
  return c.ref_policy != TNG_REF_ZERO && ((uint64_t)iter + 1) % c.ref_period == 0;
}

// Reference update from a finished decoded average (everything except what tng_step fuses into
// its decode kernel for the last-average policy).
tng_status update_reference_impl(tng_ctx* ctx, uint32_t iter, const float* vbar, float* gref) {
  const tng_config& c = ctx->cfg;
  if (c.ref_policy == TNG_REF_LAST_AVG) {
    if (!refresh_now(c, iter)) return TNG_OK;
    return tng::launch_copy_f32(gref, vbar, c.d, ctx->stream) == hipSuccess ? TNG_OK : TNG_ERR_HIP;
  }
  if (c.ref_policy == TNG_REF_WINDOW_AVG) {
    if (ctx->history == nullptr) return TNG_ERR_BAD_STATE;
    const uint32_t slot = iter % c.ref_window;
    if (tng::launch_copy_f32(ctx->history + (uint64_t)slot * c.d, vbar, c.d, ctx->stream) != hipSuccess)
      return TNG_ERR_HIP;
    if (!refresh_now(c, iter)) return TNG_OK;
    return tng::launch_window_mean(ctx->history, c.ref_window, (slot + 1) % c.ref_window, c.d, gref, ctx->stream) ==
                   hipSuccess
               ? TNG_OK
               : TNG_ERR_HIP;
  }
  return TNG_OK;
}

inline tng_status hip_status(hipError_t e) { return e == hipSuccess ? TNG_OK : TNG_ERR_HIP; }

// Device address of the static scratch array on the current device: every GPU holds its own copy at its
// own address, looked up once per device (the first call on it) and kept.
constexpr int kMaxDevices = 64;
std::mutex static_scratch_mutex;
float* static_scratch_ptr[kMaxDevices] = {};

tng_status static_scratch(float** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return TNG_ERR_HIP;
  std::lock_guard<std::mutex> lock(static_scratch_mutex);
  if (static_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return TNG_ERR_HIP;
    static_scratch_ptr[dev] = static_cast<float*>(p);
  }
  *out = static_scratch_ptr[dev];
  return TNG_OK;
}

tng::LogregData logreg_tables(const tng_ctx* ctx) {
  const uint32_t M = ctx->cfg.M;
  tng::LogregData p{};
  const void** t = ctx->tables;
  p.X = reinterpret_cast<const float* const*>(t);
  p.rowptr = reinterpret_cast<const int64_t* const*>(t);
  p.col = reinterpret_cast<const int32_t* const*>(t + M);
  p.val = reinterpret_cast<const float* const*>(t + 2 * (size_t)M);
  p.y = reinterpret_cast<const float* const*>(t + 3 * (size_t)M);
  p.n_rows = reinterpret_cast<const uint64_t*>(t + 4 * (size_t)M);
  p.tile_index = ctx->have_index ? reinterpret_cast<const uint32_t* const*>(t + 5 * (size_t)M) : nullptr;
  p.pairs = ctx->csr_pairs;
  return p;
}

bool needs_ref(const tng_config& c) { return c.norm != TNG_NORM_NONE && c.norm != TNG_NORM_MEAN; }

inline void mark(tng_ctx* ctx, uint64_t call, int which) {
  if (ctx->prof_slots != 0) (void)hipEventRecord(ctx->prof[5 * (call % ctx->prof_slots) + which], ctx->stream);
}

// The single-workgroup path for tiny problems (see launch_single_pass).  Not taken while timing events
// are recorded: they mark the separate passes.
bool single_pass_ok(const tng_ctx* ctx, const float* g, const float* gref, const float* vbar, const float* w,
                    const float* ref_out) {
  return ctx->prof_slots == 0 && tng::single_pass_applies(ctx->shape, g, gref, ctx->gref2, vbar, w, ref_out);
}

// fused_rows > 0: a gradient kernel has already left that many rows of partial maxima in the
// workspace, only their reduction remains of the scale pass.
tng_status encode_impl(tng_ctx* ctx, uint32_t iter, const float* g, const float* gref, uint32_t* codes,
                       float* scales, uint32_t fused_rows = 0) {
  if (fused_rows == 0 && single_pass_ok(ctx, g, gref, nullptr, nullptr, nullptr))  // tiny problems: one launch
    return hip_status(tng::launch_single_pass(ctx->shape, iter, g, gref, ctx->gref2, scales, codes, false, nullptr,
                                              nullptr, 0.f, nullptr, ctx->stream));
  const uint64_t call = ctx->enc_calls++;
  mark(ctx, call, 0);
  hipError_t e = hipSuccess;
  bool by_candidates = false;
  const bool mean_ref = ctx->cfg.norm == TNG_NORM_MEAN;
  if (mean_ref) {  // the worker's own reference comes first; the maximum of |g - mu| comes out of the same pass
    e = tng::launch_worker_means(ctx->shape, g, ctx->sums, ctx->shape.means,
                                 ctx->cfg.scale == TNG_SCALE_MAX ? scales : nullptr, ctx->stream);
    if (e != hipSuccess) return TNG_ERR_HIP;
  }
  if (mean_ref && ctx->cfg.scale == TNG_SCALE_MAX) {
    // nothing left of the scale pass
  } else if (ctx->cfg.scale == TNG_SCALE_L2) {
    e = tng::launch_l2_scales(ctx->shape, g, gref, ctx->gref2, ctx->sums, scales, ctx->stream);
  } else if (fused_rows > 0) {
    // the reduction of the fused partial maxima is left to the quantise launch
  } else if (ctx->cand != nullptr && tng::candidates_apply(ctx->shape, g, gref, ctx->gref2, codes)) {
    // long rows of ternary codes: the scale pass also picks out the elements that can code non-zero, and the
    // quantise pass works from those instead of reading g again
    by_candidates = true;
    e = tng::launch_absmax_candidates(ctx->shape, iter, g, gref, ctx->gref2, ctx->partials, ctx->cand, scales,
                                      ctx->stream);
  } else {
    e = tng::launch_absmax(ctx->shape, g, gref, ctx->gref2, ctx->partials, scales, ctx->stream);
  }
  if (e != hipSuccess) return TNG_ERR_HIP;
  mark(ctx, call, 1);
  const bool fused = fused_rows > 0 && !mean_ref && ctx->cfg.scale == TNG_SCALE_MAX;
  if (by_candidates)
    e = tng::launch_quantize_candidates(ctx->shape, iter, g, gref, ctx->gref2, scales, ctx->cand, codes, ctx->stream);
  else
    e = tng::launch_quantize_pack(ctx->shape, iter, g, gref, ctx->gref2, scales, codes, ctx->partials,
                                  fused ? fused_rows : 0u, ctx->stream);
  mark(ctx, call, 2);
  return hip_status(e);
}

tng_status decode_impl(tng_ctx* ctx, const uint32_t* codes, const float* scales, const float* gref, float* vbar,
                       float* w, float* ref_out) {
  const uint64_t call = ctx->dec_calls++;
  mark(ctx, call, 3);
  const hipError_t e = tng::launch_decode(ctx->shape, codes, scales, gref, ctx->gref2, vbar, w, ctx->cfg.lr,
                                          ref_out, ctx->stream);
  mark(ctx, call, 4);
  return hip_status(e);
}

tng_status check_codec_args(const tng_ctx* ctx, const float* g, const float* gref, const void* codes,
                            const float* scales, const float* vbar, bool need_g, bool need_vbar) {
  if (ctx == nullptr || codes == nullptr || scales == nullptr) return TNG_ERR_INVALID_ARG;
  if (need_g && g == nullptr) return TNG_ERR_INVALID_ARG;
  if (need_vbar && vbar == nullptr) return TNG_ERR_INVALID_ARG;
  if (needs_ref(ctx->cfg) && gref == nullptr) return TNG_ERR_INVALID_ARG;
  if (!aligned(g, 16) || !aligned(gref, 16) || !aligned(vbar, 16)) return TNG_ERR_INVALID_ARG;
  if (!aligned(codes, 4) || !aligned(scales, 4)) return TNG_ERR_INVALID_ARG;
  if (ctx->cfg.norm == TNG_NORM_COMB && ctx->gref2 == nullptr) return TNG_ERR_BAD_STATE;
  if (ctx->cfg.norm == TNG_NORM_MEAN && ctx->shape.means == nullptr) return TNG_ERR_BAD_STATE;
  return TNG_OK;
}

tng_status local_grad_impl(tng_ctx* ctx, uint32_t iter, const float* w, float* g, const tng::ScaleFusion* fuse,
                           uint32_t* fused_rows) {
  if (fused_rows != nullptr) *fused_rows = 0;
  const tng_config& c = ctx->cfg;
  const uint32_t k0 = ctx->shape.k0, k1 = ctx->shape.k1;
  hipError_t e = hipSuccess;
  switch (c.problem) {
    case TNG_PROB_LOGREG_DENSE: {
      if (!ctx->have_dense) return TNG_ERR_BAD_STATE;
      const tng::LogregData p = logreg_tables(ctx);
      e = tng::launch_logreg_dense_grad(p, c.d, c.M, c.batch, c.l2, k0, k1, iter, ctx->idx, ctx->resid, ctx->parts, w, g, fuse,
                                        fused_rows, ctx->stream);
      return hip_status(e);
    }
    case TNG_PROB_LOGREG_CSR: {
      if (!ctx->have_csr) return TNG_ERR_BAD_STATE;
      const tng::LogregData p = logreg_tables(ctx);
      e = tng::launch_minibatch_indices(k0, k1, iter, c.M, c.batch, p.n_rows, ctx->idx, ctx->stream);
      if (e != hipSuccess) return TNG_ERR_HIP;
      e = tng::launch_logreg_csr_grad(p, c.d, c.M, c.batch, c.l2, ctx->idx, ctx->rowbase, ctx->bounds, ctx->zpart,
                                      ctx->resid, w, g, fuse, fused_rows, ctx->stream);
      return hip_status(e);
    }
    case TNG_PROB_ROSENBROCK:
      e = tng::launch_rosenbrock_grad(c.d, c.M, w, ctx->noise, tng::NoiseGen{ctx->noise_sigma, k0, k1, iter}, g, fuse,
                                      fused_rows, ctx->stream);
      return hip_status(e);
    default:
      return TNG_ERR_BAD_STATE;
  }
}

void set_shape(tng_ctx* ctx, const tng_config* cfg) { ctx->shape = shape_of(cfg); }

tng_status upload_tables(tng_ctx* ctx, const void* const* t0, const void* const* t1, const void* const* t2,
                         const void* const* t3, const uint64_t* n_rows) {
  const uint32_t M = ctx->cfg.M;
  std::vector<const void*> host(5 * (size_t)M, nullptr);
  for (uint32_t m = 0; m < M; ++m) {
    if (n_rows[m] == 0 || n_rows[m] >= (1ull << 32)) return TNG_ERR_INVALID_ARG;
    if (t0[m] == nullptr || t3[m] == nullptr) return TNG_ERR_INVALID_ARG;
    if (t1 != nullptr && (t1[m] == nullptr || t2[m] == nullptr)) return TNG_ERR_INVALID_ARG;
    host[m] = t0[m];
    host[M + m] = t1 ? t1[m] : nullptr;
    host[2 * (size_t)M + m] = t2 ? t2[m] : nullptr;
    host[3 * (size_t)M + m] = t3[m];
    static_assert(sizeof(void*) == sizeof(uint64_t), "pointer tables and row counts share one array");
    host[4 * (size_t)M + m] = reinterpret_cast<const void*>(static_cast<uintptr_t>(n_rows[m]));
  }
  if (hipMemcpyAsync(ctx->tables, host.data(), host.size() * sizeof(void*), hipMemcpyHostToDevice,
                     ctx->stream) != hipSuccess)
    return TNG_ERR_HIP;
  if (hipStreamSynchronize(ctx->stream) != hipSuccess) return TNG_ERR_HIP;
  ctx->n_rows.assign(n_rows, n_rows + M);
  ctx->have_index = false;  // an index belongs to the shards it was built from
  return TNG_OK;
}

}  // namespace

extern "C" {

uint64_t tng_words_per_row(uint64_t d, uint32_t bits) {
  if (bits != 2 && bits != 4) return 0;
  const uint64_t per = 32 / bits;
  return (d + per - 1) / per;
}

size_t tng_workspace_bytes(const tng_config* cfg) {
  if (!config_valid(cfg)) return 0;
  return partition(cfg).total;
}

const char* tng_status_string(tng_status s) {
  switch (s) {
    case TNG_OK: return "ok";
    case TNG_ERR_INVALID_ARG: return "invalid argument";
    case TNG_ERR_BAD_STATE: return "call not valid in this state (problem data missing or wrong problem kind)";
    case TNG_ERR_WORKSPACE: return "workspace too small or misaligned";
    case TNG_ERR_UNSUPPORTED: return "unsupported";
    case TNG_ERR_HIP: return "HIP runtime error";
    case TNG_ERR_HOST_MEMORY: return "host memory exhausted";
    case TNG_ERR_TOO_LARGE: return "more workers than the fixed scratch of the no-allocation entry point holds";
  }
  return "unknown status";
}

tng_status tng_create(const tng_config* cfg, void* workspace, size_t workspace_bytes, void* hip_stream,
                      tng_ctx** out) {
  if (out == nullptr) return TNG_ERR_INVALID_ARG;
  *out = nullptr;
  if (!config_valid(cfg)) return TNG_ERR_INVALID_ARG;
  const Partition p = partition(cfg);
  if (workspace == nullptr || !aligned(workspace, kAlign) || workspace_bytes < p.total) return TNG_ERR_WORKSPACE;
  tng_ctx* ctx = new (std::nothrow) tng_ctx();
  if (ctx == nullptr) return TNG_ERR_HOST_MEMORY;
  ctx->cfg = *cfg;
  ctx->stream = static_cast<hipStream_t>(hip_stream);
  set_shape(ctx, cfg);
  char* base = static_cast<char*>(workspace);
  ctx->idx = reinterpret_cast<uint32_t*>(base + p.idx_off);
  ctx->resid = reinterpret_cast<float*>(base + p.resid_off);
  ctx->tables = reinterpret_cast<const void**>(base + p.tables_off);
  ctx->partials = reinterpret_cast<float*>(base + p.partials_off);
  ctx->rowbase = reinterpret_cast<int64_t*>(base + p.rowbase_off);
  ctx->bounds = reinterpret_cast<uint32_t*>(base + p.bounds_off);
  ctx->zpart = reinterpret_cast<float*>(base + p.zpart_off);
  ctx->sums = reinterpret_cast<double*>(base + p.sums_off);
  ctx->check = reinterpret_cast<uint32_t*>(base + p.check_off);
  ctx->parts = p.cand_off > p.parts_off ? reinterpret_cast<float*>(base + p.parts_off) : nullptr;
  ctx->cand = p.cand_bytes != 0 ? static_cast<void*>(base + p.cand_off) : nullptr;
  ctx->have_dense = ctx->have_csr = false;
  ctx->have_index = false;
  ctx->csr_pairs = false;
  ctx->noise = nullptr;
  ctx->noise_sigma = 0.f;
  ctx->gref2 = nullptr;
  ctx->history = nullptr;
  ctx->prof_slots = 0;
  ctx->enc_calls = ctx->dec_calls = 0;
  *out = ctx;
  return TNG_OK;
}

tng_status tng_destroy(tng_ctx* ctx) {
  if (ctx == nullptr) return TNG_ERR_INVALID_ARG;
  delete ctx;
  return TNG_OK;
}

tng_status tng_set_logreg_dense(tng_ctx* ctx, const float* const* X, const float* const* y,
                                const uint64_t* n_rows) {
  if (ctx == nullptr || X == nullptr || y == nullptr || n_rows == nullptr) return TNG_ERR_INVALID_ARG;
  if (ctx->cfg.problem != TNG_PROB_LOGREG_DENSE) return TNG_ERR_BAD_STATE;
  for (uint32_t m = 0; m < ctx->cfg.M; ++m)
    if (!aligned(X[m], 16)) return TNG_ERR_INVALID_ARG;
  const tng_status s = upload_tables(ctx, reinterpret_cast<const void* const*>(X), nullptr, nullptr,
                                     reinterpret_cast<const void* const*>(y), n_rows);
  if (s == TNG_OK) ctx->have_dense = true;
  return s;
}

tng_status tng_set_logreg_csr(tng_ctx* ctx, const int64_t* const* rowptr, const int32_t* const* col,
                              const float* const* val, const float* const* y, const uint64_t* n_rows) {
  if (ctx == nullptr || rowptr == nullptr || col == nullptr || val == nullptr || y == nullptr ||
      n_rows == nullptr)
    return TNG_ERR_INVALID_ARG;
  if (ctx->cfg.problem != TNG_PROB_LOGREG_CSR) return TNG_ERR_BAD_STATE;
  const tng_status s = upload_tables(ctx, reinterpret_cast<const void* const*>(rowptr),
                                     reinterpret_cast<const void* const*>(col),
                                     reinterpret_cast<const void* const*>(val),
                                     reinterpret_cast<const void* const*>(y), n_rows);
  if (s == TNG_OK) {
    ctx->have_csr = true;
    ctx->csr_pairs = false;
  }
  return s;
}

tng_status tng_set_logreg_csr_pairs(tng_ctx* ctx, const int64_t* const* rowptr, const tng_csr_entry* const* entries,
                                    const float* const* y, const uint64_t* n_rows) {
  if (ctx == nullptr || rowptr == nullptr || entries == nullptr || y == nullptr || n_rows == nullptr)
    return TNG_ERR_INVALID_ARG;
  if (ctx->cfg.problem != TNG_PROB_LOGREG_CSR) return TNG_ERR_BAD_STATE;
  for (uint32_t m = 0; m < ctx->cfg.M; ++m)
    if (!aligned(entries[m], 8)) return TNG_ERR_INVALID_ARG;
  // the pairs take the place of the column array; the value slot repeats the pointer so that the
  // common table check (no null entries) applies unchanged
  const tng_status s = upload_tables(ctx, reinterpret_cast<const void* const*>(rowptr),
                                     reinterpret_cast<const void* const*>(entries),
                                     reinterpret_cast<const void* const*>(entries),
                                     reinterpret_cast<const void* const*>(y), n_rows);
  if (s == TNG_OK) {
    ctx->have_csr = true;
    ctx->csr_pairs = true;
  }
  return s;
}

size_t tng_csr_index_bytes(const tng_config* cfg, const uint64_t* n_rows) {
  if (!config_valid(cfg) || cfg->problem != TNG_PROB_LOGREG_CSR || n_rows == nullptr) return 0;
  const size_t per_row = ((size_t)tng::csr_tiles(cfg->d) + 1) * sizeof(uint32_t);
  size_t total = 0;
  for (uint32_t m = 0; m < cfg->M; ++m) {
    if (n_rows[m] == 0 || n_rows[m] > 0x7fffffffull) return 0;
    total += round_up((size_t)n_rows[m] * per_row);
  }
  return total;
}

tng_status tng_set_csr_index(tng_ctx* ctx, void* index, size_t bytes) {
  if (ctx == nullptr || index == nullptr || !aligned(index, kAlign)) return TNG_ERR_INVALID_ARG;
  if (ctx->cfg.problem != TNG_PROB_LOGREG_CSR || !ctx->have_csr) return TNG_ERR_BAD_STATE;
  const size_t need = tng_csr_index_bytes(&ctx->cfg, ctx->n_rows.data());
  if (need == 0) return TNG_ERR_UNSUPPORTED;
  if (bytes < need) return TNG_ERR_WORKSPACE;
  const uint32_t M = ctx->cfg.M;
  const size_t per_row = ((size_t)tng::csr_tiles(ctx->cfg.d) + 1) * sizeof(uint32_t);
  std::vector<const void*> host(M);
  uint64_t max_rows = 0;
  size_t off = 0;
  for (uint32_t m = 0; m < M; ++m) {
    host[m] = static_cast<char*>(index) + off;
    off += round_up((size_t)ctx->n_rows[m] * per_row);
    if (ctx->n_rows[m] > max_rows) max_rows = ctx->n_rows[m];
  }
  if (hipMemcpyAsync(ctx->tables + 5 * (size_t)M, host.data(), M * sizeof(void*), hipMemcpyHostToDevice,
                     ctx->stream) != hipSuccess)
    return TNG_ERR_HIP;
  if (hipStreamSynchronize(ctx->stream) != hipSuccess) return TNG_ERR_HIP;
  ctx->have_index = true;
  const tng::LogregData p = logreg_tables(ctx);
  if (tng::launch_csr_tile_index(p, ctx->cfg.d, M, max_rows, ctx->stream) != hipSuccess) {
    ctx->have_index = false;
    return TNG_ERR_HIP;
  }
  return TNG_OK;
}

tng_status tng_validate_csr(tng_ctx* ctx, const uint64_t* nnz) {
  if (ctx == nullptr || nnz == nullptr) return TNG_ERR_INVALID_ARG;
  if (ctx->cfg.problem != TNG_PROB_LOGREG_CSR || !ctx->have_csr) return TNG_ERR_BAD_STATE;
  const uint32_t M = ctx->cfg.M;
  uint64_t* nnz_dev = reinterpret_cast<uint64_t*>(reinterpret_cast<char*>(ctx->check) + 256);
  uint64_t max_rows = 0;
  for (uint32_t m = 0; m < M; ++m) max_rows = ctx->n_rows[m] > max_rows ? ctx->n_rows[m] : max_rows;
  uint32_t flag = 0;
  auto read_flag = [&]() {
    return hipMemcpyAsync(&flag, ctx->check, sizeof(flag), hipMemcpyDeviceToHost, ctx->stream) == hipSuccess &&
           hipStreamSynchronize(ctx->stream) == hipSuccess;
  };
  if (hipMemcpyAsync(nnz_dev, nnz, M * sizeof(uint64_t), hipMemcpyHostToDevice, ctx->stream) != hipSuccess)
    return TNG_ERR_HIP;
  if (tng::launch_fill_u32(ctx->check, 1, 0u, ctx->stream) != hipSuccess) return TNG_ERR_HIP;
  const tng::LogregData p = logreg_tables(ctx);
  if (tng::launch_csr_validate_rowptr(p, M, max_rows, nnz_dev, ctx->check, ctx->stream) != hipSuccess)
    return TNG_ERR_HIP;
  if (!read_flag()) return TNG_ERR_HIP;
  if (flag != 0) return TNG_ERR_INVALID_ARG;  // the column ids are not looked at: the row pointers cannot be trusted
  if (tng::launch_csr_validate_cols(p, ctx->cfg.d, M, max_rows, ctx->check, ctx->stream) != hipSuccess)
    return TNG_ERR_HIP;
  if (!read_flag()) return TNG_ERR_HIP;
  return flag != 0 ? TNG_ERR_INVALID_ARG : TNG_OK;
}

tng_status tng_set_noise(tng_ctx* ctx, const float* noise) {
  if (ctx == nullptr || !aligned(noise, 16)) return TNG_ERR_INVALID_ARG;
  if (ctx->cfg.problem != TNG_PROB_ROSENBROCK) return TNG_ERR_BAD_STATE;
  ctx->noise = noise;
  ctx->noise_sigma = 0.f;
  return TNG_OK;
}

tng_status tng_set_noise_variance(tng_ctx* ctx, float variance) {
  if (ctx == nullptr || !(variance >= 0.0f) || !std::isfinite(variance)) return TNG_ERR_INVALID_ARG;
  if (ctx->cfg.problem != TNG_PROB_ROSENBROCK) return TNG_ERR_BAD_STATE;
  ctx->noise_sigma = std::sqrt(variance);
  if (variance > 0.0f) ctx->noise = nullptr;
  return TNG_OK;
}

tng_status tng_set_reference_history(tng_ctx* ctx, float* history) {
  if (ctx == nullptr || history == nullptr || !aligned(history, 16)) return TNG_ERR_INVALID_ARG;
  if (ctx->cfg.ref_policy != TNG_REF_WINDOW_AVG) return TNG_ERR_BAD_STATE;
  ctx->history = history;
  return TNG_OK;
}

tng_status tng_set_second_reference(tng_ctx* ctx, const float* gref2) {
  if (ctx == nullptr || gref2 == nullptr || !aligned(gref2, 16)) return TNG_ERR_INVALID_ARG;
  ctx->gref2 = gref2;
  return TNG_OK;
}

tng_status tng_set_worker_means(tng_ctx* ctx, float* means) {
  if (ctx == nullptr || means == nullptr || !aligned(means, 4)) return TNG_ERR_INVALID_ARG;
  if (ctx->cfg.norm != TNG_NORM_MEAN) return TNG_ERR_BAD_STATE;
  ctx->shape.means = means;
  return TNG_OK;
}

tng_status tng_set_profile_events(tng_ctx* ctx, void* const* events, uint32_t slots) {
  if (ctx == nullptr || (events == nullptr && slots != 0)) return TNG_ERR_INVALID_ARG;
  ctx->prof.clear();
  ctx->prof_slots = 0;
  ctx->enc_calls = ctx->dec_calls = 0;
  if (events == nullptr || slots == 0) return TNG_OK;
  for (size_t i = 0; i < 5 * (size_t)slots; ++i) {
    if (events[i] == nullptr) {
      ctx->prof.clear();
      return TNG_ERR_INVALID_ARG;
    }
    ctx->prof.push_back(static_cast<hipEvent_t>(events[i]));
  }
  ctx->prof_slots = slots;
  return TNG_OK;
}

tng_status tng_rng_draws(tng_ctx* ctx, uint32_t iter, uint32_t worker, uint32_t stream, uint64_t first,
                         uint64_t count, uint32_t* out) {
  if (ctx == nullptr || (out == nullptr && count != 0) || !aligned(out, 4)) return TNG_ERR_INVALID_ARG;
  if (first + count < first || ((first + count) >> 2) > (1ull << 32)) return TNG_ERR_INVALID_ARG;
  return hip_status(tng::launch_rng_draws(ctx->shape.k0, ctx->shape.k1, iter, worker, stream, first, count, out,
                                          ctx->stream));
}

tng_status tng_minibatch_indices(tng_ctx* ctx, uint32_t iter, uint32_t* idx) {
  if (ctx == nullptr || idx == nullptr || !aligned(idx, 4)) return TNG_ERR_INVALID_ARG;
  if (!ctx->have_dense && !ctx->have_csr) return TNG_ERR_BAD_STATE;
  const tng::LogregData p = logreg_tables(ctx);
  return hip_status(tng::launch_minibatch_indices(ctx->shape.k0, ctx->shape.k1, iter, ctx->cfg.M,
                                                  ctx->cfg.batch, p.n_rows, idx, ctx->stream));
}

tng_status tng_local_grad(tng_ctx* ctx, uint32_t iter, const float* w, float* g) {
  if (ctx == nullptr || w == nullptr || g == nullptr || !aligned(w, 16) || !aligned(g, 16))
    return TNG_ERR_INVALID_ARG;
  return local_grad_impl(ctx, iter, w, g, nullptr, nullptr);
}

tng_status tng_normalize_encode(tng_ctx* ctx, uint32_t iter, const float* g, const float* gref,
                                uint32_t* codes, float* scales) {
  const tng_status s = check_codec_args(ctx, g, gref, codes, scales, nullptr, true, false);
  if (s != TNG_OK) return s;
  return encode_impl(ctx, iter, g, gref, codes, scales);
}

tng_status tng_normalize_encode_static(const tng_config* cfg, void* hip_stream, uint32_t iter, const float* g,
                                       const float* gref, uint32_t* codes, float* scales) {
  if (!config_valid(cfg)) return TNG_ERR_INVALID_ARG;
  if (cfg->scale != TNG_SCALE_MAX ||
      (cfg->norm != TNG_NORM_NONE && cfg->norm != TNG_NORM_SUB && cfg->norm != TNG_NORM_QUOT))
    return TNG_ERR_UNSUPPORTED;
  if (cfg->M > kStaticMaxWorkers) return TNG_ERR_TOO_LARGE;
  tng_ctx local{};  // a host object on the stack; its vectors stay empty
  local.cfg = *cfg;
  local.stream = static_cast<hipStream_t>(hip_stream);
  set_shape(&local, cfg);
  const tng_status s = check_codec_args(&local, g, gref, codes, scales, nullptr, true, false);
  if (s != TNG_OK) return s;
  const tng_status sp = static_scratch(&local.partials);
  if (sp != TNG_OK) return sp;
  // nothing in the scratch has to start at zero: the scale pass writes every partial maximum that its
  // reduction reads
  return encode_impl(&local, iter, g, gref, codes, scales);
}

tng_status tng_decode_aggregate(tng_ctx* ctx, const uint32_t* codes, const float* scales, const float* gref,
                                float* vbar) {
  const tng_status s = check_codec_args(ctx, nullptr, gref, codes, scales, vbar, false, true);
  if (s != TNG_OK) return s;
  return decode_impl(ctx, codes, scales, gref, vbar, nullptr, nullptr);
}

tng_status tng_update_reference(tng_ctx* ctx, uint32_t iter, const float* vbar, float* gref) {
  if (ctx == nullptr || vbar == nullptr || gref == nullptr || !aligned(vbar, 16) || !aligned(gref, 16))
    return TNG_ERR_INVALID_ARG;
  return update_reference_impl(ctx, iter, vbar, gref);
}

tng_status tng_step(tng_ctx* ctx, uint32_t iter, float* w, float* gref, float* g, uint32_t* codes,
                    float* scales, float* vbar) {
  if (ctx == nullptr || w == nullptr || gref == nullptr || !aligned(w, 16)) return TNG_ERR_INVALID_ARG;
  tng_status s = check_codec_args(ctx, g, gref, codes, scales, vbar, true, true);
  if (s != TNG_OK) return s;
  if (ctx->cfg.ref_policy == TNG_REF_WINDOW_AVG && ctx->history == nullptr) return TNG_ERR_BAD_STATE;
  if (ctx->cfg.problem == TNG_PROB_LOGREG_DENSE && !ctx->have_dense) return TNG_ERR_BAD_STATE;
  if (ctx->cfg.problem == TNG_PROB_LOGREG_CSR && !ctx->have_csr) return TNG_ERR_BAD_STATE;
  const tng_config& c = ctx->cfg;
  const bool window = c.ref_policy == TNG_REF_WINDOW_AVG;
  const uint32_t slot = window ? iter % c.ref_window : 0u;
  // where the decode pass leaves a second copy of the decoded average: its slot of the history ring
  // (window average), or the reference itself when it is refreshed now (last average)
  float* ref_out = window ? ctx->history + (uint64_t)slot * c.d : (refresh_now(c, iter) ? gref : nullptr);
  // tiny problems: everything after the gradient in one launch
  const bool single = single_pass_ok(ctx, g, gref, vbar, w, ref_out);
  uint32_t fused_rows = 0;
  if (c.problem != TNG_PROB_EXTERNAL) {
    const tng::ScaleFusion fuse{c.norm, c.quot_eps, gref, ctx->gref2, ctx->partials};
    // the maximum can ride along with the gradient kernel; a scale that needs the row mean or an
    // ordered sum cannot
    const bool can_fuse = !single && c.norm != TNG_NORM_MEAN && c.scale == TNG_SCALE_MAX;
    s = local_grad_impl(ctx, iter, w, g, can_fuse ? &fuse : nullptr, can_fuse ? &fused_rows : nullptr);
    if (s != TNG_OK) return s;
  }
  if (single) {
    s = hip_status(tng::launch_single_pass(ctx->shape, iter, g, gref, ctx->gref2, scales, codes, true, vbar, w, c.lr,
                                           ref_out, ctx->stream));
    if (s != TNG_OK) return s;
  } else {
    s = encode_impl(ctx, iter, g, gref, codes, scales, fused_rows);
    if (s != TNG_OK) return s;
    s = decode_impl(ctx, codes, scales, gref, vbar, w, ref_out);
    if (s != TNG_OK) return s;
  }
  if (window && refresh_now(c, iter))
    return hip_status(tng::launch_window_mean(ctx->history, c.ref_window, (slot + 1) % c.ref_window, c.d, gref,
                                              ctx->stream));
  return TNG_OK;
}

}  // extern "C"
