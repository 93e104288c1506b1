// Host-side launch interface between the C-ABI layer and the HIP kernels of libtng.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tng {

struct CodecShape {
  uint64_t d;      // elements per worker
  uint64_t words;  // packed 32-bit words per worker row
  uint32_t M;      // workers
  int bits;        // 2 or 4
  int norm;        // kNorm*
  float eps;       // clamp of the divisor reference
  uint32_t k0, k1; // Philox key (seed low, seed high)
  int scale_l2;    // 0: R = max |v|, 1: R = ||v||_2
  float* means;    // device [M]: per-worker means of the mean reference (kNormMean), else unused
};

hipError_t launch_fill_u32(uint32_t* p, uint64_t n, uint32_t value, hipStream_t s);
hipError_t launch_copy_f32(float* dst, const float* src, uint64_t n, hipStream_t s);
// out = (history[first] + history[first+1] + ... cyclically over `window` slots of d floats) * (1/window)
hipError_t launch_window_mean(const float* history, uint32_t window, uint32_t first, uint64_t d, float* out,
                              hipStream_t s);
hipError_t launch_rng_draws(uint32_t k0, uint32_t k1, uint32_t iter, uint32_t worker, uint32_t stream,
                            uint64_t first, uint64_t count, uint32_t* out, hipStream_t s);

// Workgroups (per worker group) of the scale pass; each leaves one partial maximum per worker.
constexpr uint32_t kAbsmaxMaxBlocks = 4096;

// scales[m] = max_e |normalize(g[m][e])|, 0 when below FLT_MIN.  partials: device scratch of
// kAbsmaxMaxBlocks * M floats.  Two launches: partial maxima per workgroup, then one reduction.
hipError_t launch_absmax(const CodecShape& c, const float* g, const float* gref, const float* gref2,
                         float* partials, float* scales, hipStream_t s);
// Order-pinned float64 sums per worker (4096-element chunks of 256 strided lanes, chunks in groups of
// 256, everything added in index order).  sums: device scratch of tree_sum_scratch(d, M) doubles.
// launch_worker_means: means[m] = float(sum_e g[m][e] / d); if scales != nullptr also
// scales[m] = max_e |g[m][e] - means[m]| (0 when below FLT_MIN), from the row's extremes in the same
// pass.  launch_l2_scales: scales[m] = float(sqrt(sum_e v^2)), v the normalised gradient (c.means
// must hold the means for kNormMean), 0 when below FLT_MIN.
size_t tree_sum_scratch(uint64_t d, uint32_t M);
hipError_t launch_worker_means(const CodecShape& c, const float* g, double* sums, float* means, float* scales,
                               hipStream_t s);
hipError_t launch_l2_scales(const CodecShape& c, const float* g, const float* gref, const float* gref2, double* sums,
                            float* scales, hipStream_t s);

// The ternary coder that reads g once (2-bit codes, largest-magnitude scale): the scale pass also keeps,
// per worker and tile of 1024 coordinates, the few elements that can code non-zero whatever the scale turns
// out to be (tested against a lower bound of it), and the quantise pass codes those from the slots instead
// of reading g again; same codes and scales as launch_absmax + launch_quantize_pack, bit for bit.
// candidate_scratch_bytes: device scratch needed (256-byte aligned), 0 where the path does not apply
// (other code widths, scales and normalisations, rows that are not whole tiles, small problems);
// candidates_apply: whether it may be used for these operands (scratch size non-zero, 16-byte alignment).
size_t candidate_scratch_bytes(const CodecShape& c);
bool candidates_apply(const CodecShape& c, const float* g, const float* gref, const float* gref2, const uint32_t* codes);
hipError_t launch_absmax_candidates(const CodecShape& c, uint32_t iter, const float* g, const float* gref,
                                    const float* gref2, float* partials, void* scratch, float* scales, hipStream_t s);
hipError_t launch_quantize_candidates(const CodecShape& c, uint32_t iter, const float* g, const float* gref,
                                      const float* gref2, const float* scales, void* scratch, uint32_t* codes,
                                      hipStream_t s);

// Reduction of nblocks rows of per-workgroup partial maxima (partials[block][m]) to scales[m].
hipError_t launch_absmax_finish(const float* partials, uint32_t nblocks, uint32_t M, float* scales, hipStream_t s);

// Optional fusion of the scale pass into a gradient launcher: when it can (vector path, at most
// kAbsmaxMaxBlocks workgroups per worker), its last kernel also leaves the per-workgroup maxima of
// |normalize(g)| in partials[block][m] and reports the number of rows; otherwise it reports 0 and the
// caller runs the scale pass itself.  g is then read once instead of twice per iteration.
struct ScaleFusion {
  int norm;
  float eps;
  const float* gref;
  const float* gref2;
  float* partials;
};

// fused_rows == 0: scales[m] is read.  fused_rows > 0: the scale pass was fused into a gradient kernel
// that left fused_rows rows of partial maxima in partials; scales[m] is then written as well (by the
// quantiser itself for small problems, by the reduction kernel otherwise).
hipError_t launch_quantize_pack(const CodecShape& c, uint32_t iter, const float* g, const float* gref,
                                const float* gref2, float* scales, uint32_t* codes, const float* partials,
                                uint32_t fused_rows, hipStream_t s);
// vbar = denorm(mean_m decode).  If w != nullptr also w -= lr * vbar; if ref_out != nullptr also
// ref_out = vbar (ref_out may alias gref).
hipError_t launch_decode(const CodecShape& c, const uint32_t* codes, const float* scales,
                         const float* gref, const float* gref2, float* vbar, float* w, float lr,
                         float* ref_out, hipStream_t s);

// Tiny problems (d <= 1024 and a multiple of 4, M <= 16, largest-magnitude scale, no per-worker mean,
// 16-byte aligned operands): scale, quantise and pack in ONE single-workgroup launch, and with
// decode = true the decode / average / de-normalise / update pass as well (vbar, w, ref_out as for
// launch_decode).  single_pass_applies tells whether launch_single_pass may be called.
bool single_pass_applies(const CodecShape& c, const float* g, const float* gref, const float* gref2, const float* vbar,
                         const float* w, const float* ref_out);
hipError_t launch_single_pass(const CodecShape& c, uint32_t iter, const float* g, const float* gref, const float* gref2,
                              float* scales, uint32_t* codes, bool decode, float* vbar, float* w, float lr,
                              float* ref_out, hipStream_t s);

struct LogregData {
  const float* const* X;        // device table [M] of dense shards (dense problem)
  const int64_t* const* rowptr; // device tables [M] (CSR problem)
  const int32_t* const* col;    // column ids; with pairs: the (column, value) pair arrays
  const float* const* val;      // values; unused with pairs
  bool pairs;                   // CSR entries are stored as (int32 column, float value) pairs
  const float* const* y;        // device table [M]
  const uint64_t* n_rows;       // device [M]
  const uint32_t* const* tile_index;  // device table [M] of per-row tile indices (CSR), or nullptr
};

hipError_t launch_minibatch_indices(uint32_t k0, uint32_t k1, uint32_t iter, uint32_t M, uint32_t batch,
                                    const uint64_t* n_rows, uint32_t* idx, hipStream_t s);
// The minibatch row ids of iteration iter are drawn inside (Philox key k0, k1) and left in idx.
// parts: device scratch of dense_row_splits(d, M, batch) * M * d floats (per-workgroup partial gradients of
// the one-pass kernel for wide rows), or nullptr; dense_row_splits returns 0 where that kernel does not apply.
uint32_t dense_row_splits(uint64_t d, uint32_t M, uint32_t batch);
hipError_t launch_logreg_dense_grad(const LogregData& p, uint64_t d, uint32_t M, uint32_t batch, float l2,
                                    uint32_t k0, uint32_t k1, uint32_t iter, uint32_t* idx, float* resid,
                                    float* parts, const float* w, float* g, const ScaleFusion* fuse,
                                    uint32_t* fused_rows, hipStream_t s);
// Column tiles of the CSR gradient: 2^kCsrTileShift coordinates (128 KiB of fp64 in LDS).
constexpr uint32_t kCsrTileShift = 14;
uint32_t csr_tiles(uint64_t d);
// Device scratch: rowbase int64[M][batch]; bounds uint32[M][csr_tiles(d) + 1][batch];
// zpart float[M][csr_tiles(d)][batch] (partial dot products per tile, or per pair of tiles in the
// first half of it); z float[M][batch], which receives (sigma(z_i) - y_i) / batch.
// Columns must be ascending within each row.
// p.tile_index (optional): per worker uint32[n_rows][csr_tiles(d) + 1], entry [row][t] = offset within
// the row of the first stored entry whose column is at or beyond the start of tile t; built once by
// launch_csr_tile_index.  With it the per-iteration pass over the column ids is replaced by a gather.
// Checks of the CSR shards (see the kernels): nnz device uint64[M] = entries stored per worker; flag:
// device uint32, cleared by the caller; bit 0 = bad row pointers, bit 1 = column out of [0, d),
// bit 2 = columns of a row not strictly ascending.  The column pass reads what the row pointers name,
// so it may only run after the row-pointer pass has come back clean.
hipError_t launch_csr_validate_rowptr(const LogregData& p, uint32_t M, uint64_t max_rows, const uint64_t* nnz,
                                      uint32_t* flag, hipStream_t s);
hipError_t launch_csr_validate_cols(const LogregData& p, uint64_t d, uint32_t M, uint64_t max_rows, uint32_t* flag,
                                    hipStream_t s);
hipError_t launch_csr_tile_index(const LogregData& p, uint64_t d, uint32_t M, uint64_t max_rows, hipStream_t s);
hipError_t launch_logreg_csr_grad(const LogregData& p, uint64_t d, uint32_t M, uint32_t batch, float l2,
                                  const uint32_t* idx, int64_t* rowbase, uint32_t* bounds, float* zpart, float* z,
                                  const float* w, float* g, const ScaleFusion* fuse, uint32_t* fused_rows,
                                  hipStream_t s);
// Gaussian noise made on the device (sigma > 0): element e of worker m at iteration iter is
// sigma * z, z from the Box-Muller transform of the Philox block (e >> 2, m, iter, 2): words 0, 1
// give z for e & 3 = 0 (cosine) and 1 (sine), words 2, 3 for e & 3 = 2 and 3;
// u1 = ((word >> 8) + 1) 2^-24 in (0, 1], u2 = (word >> 8) 2^-24, z = sqrt(-2 ln u1) {cos, sin}(2 pi u2).
struct NoiseGen {
  float sigma;
  uint32_t k0, k1, iter;
};
// noise: tensor [M][d] added to the gradient, or nullptr; gen.sigma > 0 adds generated noise instead
// (the tensor is then ignored).
hipError_t launch_rosenbrock_grad(uint64_t d, uint32_t M, const float* x, const float* noise, NoiseGen gen, float* g,
                                  const ScaleFusion* fuse, uint32_t* fused_rows, hipStream_t s);

}  // namespace tng
