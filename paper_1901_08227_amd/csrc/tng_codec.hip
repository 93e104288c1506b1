// Codec kernels of libtng: scale (max of the normalised gradient), stochastic quantise + pack,
// and decode + average + de-normalise (+ iterate / reference update), for gfx950.
//
// All three stream fp32 data once; they are bound by HBM bandwidth (and, for the quantiser, by the
// integer multiplies of the counter-based RNG), never by matrix math.  Layout choices:
//  * a workgroup owns a tile of coordinates and loops over the workers inside the kernel, so the
//    shared reference tile is fetched once and kept in registers;
//  * every global access is a coalesced 16-byte (fp32) or 4-byte (packed words) per-lane access;
//    the 2- or 4-bit codes a lane produces are transposed into whole words through LDS;
//  * Philox block j covers elements 4j..4j+3, i.e. exactly one float4.
#include "tng_device.hpp"
#include "tng_kernels.hpp"

#include <float.h>
#include <type_traits>

namespace tng {

namespace {

constexpr int kWavesPerBlock = kBlock / kWave;
constexpr uint32_t kFusedScaleRows = 8;  // at most this many rows of partial maxima are reduced by the quantiser itself
constexpr int kLoadsPerLane = 4;  // float4 loads per lane and worker in the quantiser tile
constexpr uint32_t kMaxGridX = 1u << 20;

__global__ __launch_bounds__(kBlock) void fill_u32_kernel(uint32_t* p, uint64_t n, uint32_t v) {
  const uint64_t stride = (uint64_t)gridDim.x * kBlock;
  for (uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += stride) p[i] = v;
}

__global__ __launch_bounds__(kBlock) void copy_f32_kernel(float* __restrict__ dst,
                                                          const float* __restrict__ src, uint64_t n) {
  const uint64_t stride = (uint64_t)gridDim.x * kBlock;
  for (uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

// Four float4 per thread in flight and one trip per workgroup wherever the grid allows: the shape that
// measured fastest for a plain copy (1 GiB: 6.4 TB/s on read + written bytes, against 5.4 with one float4 per
// thread and 16384 workgroups striding; streaming loads and stores in both).
constexpr int kCopyPerThread = 4;
__global__ __launch_bounds__(kBlock) void copy_f32x4_kernel(float4* __restrict__ dst,
                                                            const float4* __restrict__ src, uint64_t n) {
  const uint64_t stride = (uint64_t)gridDim.x * kBlock * kCopyPerThread;
  for (uint64_t i = (uint64_t)blockIdx.x * kBlock * kCopyPerThread + threadIdx.x; i < n; i += stride) {
    float4 x[kCopyPerThread];
#pragma unroll
    for (int u = 0; u < kCopyPerThread; ++u)
      if (i + (uint64_t)u * kBlock < n) x[u] = load_stream(src + i + (uint64_t)u * kBlock);
#pragma unroll
    for (int u = 0; u < kCopyPerThread; ++u)
      if (i + (uint64_t)u * kBlock < n) store_stream(dst + i + (uint64_t)u * kBlock, x[u]);
  }
}

// Window-average reference (section "Reference Vectors"): mean of the last `window` decoded
// averages, added oldest first, one rounding per addition.
__global__ __launch_bounds__(kBlock) void window_mean_kernel(const float* __restrict__ history, uint32_t window,
                                                             uint32_t first, uint64_t d, float inv_window,
                                                             float* __restrict__ out) {
  const uint64_t stride = (uint64_t)gridDim.x * kBlock;
  for (uint64_t e = (uint64_t)blockIdx.x * kBlock + threadIdx.x; e < d; e += stride) {
    float acc = 0.f;
    uint32_t slot = first;
    for (uint32_t k = 0; k < window; ++k) {
      acc = acc + history[(uint64_t)slot * d + e];
      slot = slot + 1 == window ? 0u : slot + 1;
    }
    out[e] = acc * inv_window;
  }
}

// The same, four coordinates per thread (d a multiple of 4, 16-byte aligned operands).
__global__ __launch_bounds__(kBlock) void window_mean_vec_kernel(const float4* __restrict__ history, uint32_t window,
                                                                 uint32_t first, uint64_t nvec, float inv_window,
                                                                 float4* __restrict__ out) {
  const uint64_t stride = (uint64_t)gridDim.x * kBlock;
  for (uint64_t q = (uint64_t)blockIdx.x * kBlock + threadIdx.x; q < nvec; q += stride) {
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    uint32_t slot = first;
    for (uint32_t k = 0; k < window; ++k) {
      const float4 h = load_stream(history + (uint64_t)slot * nvec + q);
      acc.x = acc.x + h.x;
      acc.y = acc.y + h.y;
      acc.z = acc.z + h.z;
      acc.w = acc.w + h.w;
      slot = slot + 1 == window ? 0u : slot + 1;
    }
    store_stream(out + q, make_float4(acc.x * inv_window, acc.y * inv_window, acc.z * inv_window, acc.w * inv_window));
  }
}

__global__ __launch_bounds__(kBlock) void rng_draws_kernel(uint32_t k0, uint32_t k1, uint32_t iter,
                                                           uint32_t worker, uint32_t stream,
                                                           uint64_t first, uint64_t count, uint32_t* out) {
  const uint64_t stride = (uint64_t)gridDim.x * kBlock;
  for (uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x; i < count; i += stride) {
    const uint64_t j = first + i;
    const U32x4 r = philox4x32_10((uint32_t)(j >> 2), worker, iter, stream, k0, k1);
    const uint32_t lane = (uint32_t)(j & 3);
    out[i] = lane == 0 ? r.x : lane == 1 ? r.y : lane == 2 ? r.z : r.w;
  }
}

// ------------------------------------------------------------------------------------------
// Reference operands of one float4 of coordinates.
// ------------------------------------------------------------------------------------------
template <int NORM>
struct RefTile {
  float4 r1, r2;
  double inv[4];  // binary64 reciprocals of the divisor (Eq. 2: r1, combined form: r2), see reciprocals()
  // STREAM: the tile is read once by this kernel (non-temporal); otherwise it is re-read soon and
  // should stay in cache.
  template <bool STREAM = true>
  __device__ __forceinline__ void load(const float4* ref, const float4* ref2, uint64_t i, float eps) {
    r1 = make_float4(0.f, 0.f, 0.f, 0.f);
    r2 = make_float4(1.f, 1.f, 1.f, 1.f);
    if (NORM == kNormSub || NORM == kNormComb) r1 = STREAM ? load_stream(ref + i) : ref[i];
    if (NORM == kNormQuot) {
      const float4 r = STREAM ? load_stream(ref + i) : ref[i];
      r1 = make_float4(clamp_ref(r.x, eps), clamp_ref(r.y, eps), clamp_ref(r.z, eps), clamp_ref(r.w, eps));
    }
    if (NORM == kNormComb) {
      const float4 r = STREAM ? load_stream(ref2 + i) : ref2[i];
      r2 = make_float4(clamp_ref(r.x, eps), clamp_ref(r.y, eps), clamp_ref(r.z, eps), clamp_ref(r.w, eps));
    }
  }
  // Every worker divides by the same clamped reference (Eq. 2 and the combined form): the scale and the
  // quantise pass take its binary64 reciprocal once per coordinate and multiply per worker
  // (quotient_by_reciprocal), 4 operations per element instead of the 12 of a division.
  __device__ __forceinline__ void reciprocals() {
    const float4& b = NORM == kNormQuot ? r1 : r2;
    if (NORM == kNormQuot || NORM == kNormComb) {
      inv[0] = 1.0 / (double)b.x;
      inv[1] = 1.0 / (double)b.y;
      inv[2] = 1.0 / (double)b.z;
      inv[3] = 1.0 / (double)b.w;
    }
  }
};

// Worth it from four workers per reference tile on: the reciprocal itself costs about two divisions.
template <int NORM, int MC>
constexpr bool kByReciprocal = (NORM == kNormQuot || NORM == kNormComb) && MC >= 4;

// The four values one float4 of a worker's row hands to the coder, the divisions of Eq. 2 / the
// combined form done through the reciprocals; the (rare) float4 with a subnormal quotient is redone
// with the division itself, so the values are those of normalize_w bit for bit.
template <int NORM, bool RECIP>
__device__ __forceinline__ float4 normalize4(const float4& x, const RefTile<NORM>& rt, float mu) {
  if (!RECIP) {
    return make_float4(normalize_w<NORM>(x.x, rt.r1.x, rt.r2.x, mu), normalize_w<NORM>(x.y, rt.r1.y, rt.r2.y, mu),
                       normalize_w<NORM>(x.z, rt.r1.z, rt.r2.z, mu), normalize_w<NORM>(x.w, rt.r1.w, rt.r2.w, mu));
  }
  float4 n = x;  // numerators
  if (NORM == kNormComb) n = make_float4(x.x - rt.r1.x, x.y - rt.r1.y, x.z - rt.r1.z, x.w - rt.r1.w);
  float4 v = make_float4(quotient_by_reciprocal(n.x, rt.inv[0]), quotient_by_reciprocal(n.y, rt.inv[1]),
                         quotient_by_reciprocal(n.z, rt.inv[2]), quotient_by_reciprocal(n.w, rt.inv[3]));
  if ((int)is_subnormal(v.x) | (int)is_subnormal(v.y) | (int)is_subnormal(v.z) | (int)is_subnormal(v.w)) {
    const float4& b = NORM == kNormQuot ? rt.r1 : rt.r2;
    v = make_float4(n.x / b.x, n.y / b.y, n.z / b.z, n.w / b.w);
  }
  return v;
}

// max |normalize4(x)| over one float4.  The maximum is taken in binary64 and rounded once (rounding is
// monotone, so this is the maximum of the rounded quotients); it is right whenever it is 0 or at least
// 2^-125, because then the largest quotient is of normal size and every subnormal one lies below it.
template <int NORM>
__device__ __forceinline__ double absmax4_by_reciprocal(const float4& x, const RefTile<NORM>& rt) {
  float4 n = x;
  if (NORM == kNormComb) n = make_float4(x.x - rt.r1.x, x.y - rt.r1.y, x.z - rt.r1.z, x.w - rt.r1.w);
  const double q0 = fabs((double)n.x * rt.inv[0]), q1 = fabs((double)n.y * rt.inv[1]);
  const double q2 = fabs((double)n.z * rt.inv[2]), q3 = fabs((double)n.w * rt.inv[3]);
  return fmax(fmax(q0, q1), fmax(q2, q3));
}

template <int NORM>
__device__ __forceinline__ void load_ref_scalar(const float* ref, const float* ref2, uint64_t e, float eps,
                                                float& r1, float& r2) {
  r1 = 0.f;
  r2 = 1.f;
  if (NORM == kNormSub || NORM == kNormComb) r1 = ref[e];
  if (NORM == kNormQuot) r1 = clamp_ref(ref[e], eps);
  if (NORM == kNormComb) r2 = clamp_ref(ref2[e], eps);
}

// Block maximum of MC per-thread values, written to this workgroup's slot of the partial-maxima
// array (partials[blockIdx.x][m]); a second, tiny kernel reduces the slots.  Thousands of atomic
// maxima on the same few words serialise in L2 (about 10 ns each), plain stores do not.
template <int MC>
__device__ __forceinline__ void block_max_to_partials(float (&mx)[MC], uint32_t m0, uint32_t M, float* partials) {
  __shared__ float red[MC][kWavesPerBlock];
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
#pragma unroll
  for (int mm = 0; mm < MC; ++mm) {
    const float v = wave_max(mx[mm]);
    if (lane == 0) red[mm][wave] = v;
  }
  __syncthreads();
  if (threadIdx.x < MC && m0 + threadIdx.x < M) {
    float v = red[threadIdx.x][0];
#pragma unroll
    for (int k = 1; k < kWavesPerBlock; ++k) v = fmaxf(v, red[threadIdx.x][k]);
    partials[(uint64_t)blockIdx.x * M + m0 + threadIdx.x] = v;
  }
}

// scales[m] = max over the nblocks partial maxima of worker m; a maximum below the smallest normal
// number is taken as 0.  One workgroup per worker.
__device__ __forceinline__ void absmax_finish_worker(const float* __restrict__ partials, uint32_t nblocks, uint32_t M,
                                                     float* __restrict__ scales, uint32_t m) {
  __shared__ float red[kWavesPerBlock];
  float v = 0.f;
  for (uint32_t b = threadIdx.x; b < nblocks; b += kBlock) v = fmaxf(v, partials[(uint64_t)b * M + m]);
  v = wave_max(v);
  if (threadIdx.x % kWave == 0) red[threadIdx.x / kWave] = v;
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int k = 1; k < kWavesPerBlock; ++k) v = fmaxf(v, red[k]);
    scales[m] = v < FLT_MIN ? 0.f : v;
  }
}
__global__ __launch_bounds__(kBlock) void absmax_finish_kernel(const float* __restrict__ partials, uint32_t nblocks,
                                                               uint32_t M, float* __restrict__ scales) {
  absmax_finish_worker(partials, nblocks, M, scales, blockIdx.x);
}

// The M gradient rows as the vector kernels read them.  Row m starts m * pitch floats into the array;
// the pitch (= d) need not be a multiple of 4, so a row may start at any 4-byte boundary (hence the
// 16-byte loads that assume 4-byte alignment only).
struct GradRows {
  const float* base;
  uint64_t pitch;
  __device__ __forceinline__ const v4f_u_t* row(uint32_t m) const {
    return reinterpret_cast<const v4f_u_t*>(base + (uint64_t)m * pitch);
  }
};
__device__ __forceinline__ float4 load_row_stream(const v4f_u_t* p) {
  const v4f_u_t v = __builtin_nontemporal_load(p);
  return make_float4(v.x, v.y, v.z, v.w);
}

// ------------------------------------------------------------------------------------------
// Pass 1: R_m = max_e |v_{m,e}|   (section "Gradient Compression": R = max_d |v_d|)
// ------------------------------------------------------------------------------------------
// A wavefront owns kAbsmaxLoads * 64 consecutive float4 (4 KiB) of every worker row and walks the
// workers one after the other with the next worker's four loads in flight; reading one row at a
// time (instead of all rows at once) and streaming loads measured ~20 % faster on HBM.  The
// reference tile stays in registers.
constexpr int kAbsmaxLoads = 4;

template <int NORM, bool FULL>
__device__ __forceinline__ void absmax_load(const v4f_u_t* __restrict__ row, const uint64_t (&iv)[kAbsmaxLoads],
                                            uint64_t nvec, float4 (&x)[kAbsmaxLoads]) {
#pragma unroll
  for (int j = 0; j < kAbsmaxLoads; ++j) {
    if (FULL || iv[j] < nvec) {
      x[j] = load_row_stream(row + iv[j]);
    } else {
      x[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
  }
}

template <int NORM, bool FULL, bool RECIP>
__device__ __forceinline__ float absmax_reduce(const float4 (&x)[kAbsmaxLoads], const RefTile<NORM> (&rt)[kAbsmaxLoads],
                                               const uint64_t (&iv)[kAbsmaxLoads], uint64_t nvec, float mu) {
  if (RECIP) {
    double mx64 = 0.0;
#pragma unroll
    for (int j = 0; j < kAbsmaxLoads; ++j) {
      if (FULL || iv[j] < nvec) mx64 = fmax(mx64, absmax4_by_reciprocal<NORM>(x[j], rt[j]));
    }
    if (!(mx64 > 0.0 && mx64 < 0x1p-125)) return (float)mx64;
    // else (a tile whose quotients are all tiny): once more with the divisions themselves
  }
  float mx = 0.f;
#pragma unroll
  for (int j = 0; j < kAbsmaxLoads; ++j) {
    if (FULL || iv[j] < nvec) {
      const float a0 = fabsf(normalize_w<NORM>(x[j].x, rt[j].r1.x, rt[j].r2.x, mu));
      const float a1 = fabsf(normalize_w<NORM>(x[j].y, rt[j].r1.y, rt[j].r2.y, mu));
      const float a2 = fabsf(normalize_w<NORM>(x[j].z, rt[j].r1.z, rt[j].r2.z, mu));
      const float a3 = fabsf(normalize_w<NORM>(x[j].w, rt[j].r1.w, rt[j].r2.w, mu));
      mx = fmaxf(mx, fmaxf(fmaxf(a0, a1), fmaxf(a2, a3)));
    }
  }
  return mx;
}

template <int NORM, int MC, bool FULL>
__device__ __forceinline__ void absmax_rows(const GradRows& g, const RefTile<NORM> (&rt)[kAbsmaxLoads],
                                            const uint64_t (&iv)[kAbsmaxLoads], uint64_t nvec, uint32_t m0,
                                            uint32_t M, const float* __restrict__ means, float (&mx)[MC]) {
  constexpr int L = kAbsmaxLoads;
  float4 xa[L], xb[L];
  // rows past M (only when MC does not divide M) repeat the last row, which leaves its maximum unchanged
  auto row = [&](int mm) { return g.row(min(m0 + (uint32_t)mm, M - 1)); };
  auto mean_of = [&](int mm) { return NORM == kNormMean ? means[min(m0 + (uint32_t)mm, M - 1)] : 0.f; };
  absmax_load<NORM, FULL>(row(0), iv, nvec, xa);
#pragma unroll
  for (int mm = 0; mm < MC; mm += 2) {
    if (mm + 1 < MC) absmax_load<NORM, FULL>(row(mm + 1), iv, nvec, xb);
    mx[mm] = fmaxf(mx[mm], absmax_reduce<NORM, FULL, kByReciprocal<NORM, MC>>(xa, rt, iv, nvec, mean_of(mm)));
    if (mm + 1 < MC) {
      if (mm + 2 < MC) absmax_load<NORM, FULL>(row(mm + 2), iv, nvec, xa);
      mx[mm + 1] = fmaxf(mx[mm + 1], absmax_reduce<NORM, FULL, kByReciprocal<NORM, MC>>(xb, rt, iv, nvec, mean_of(mm + 1)));
    }
  }
}

template <int NORM, int MC>
__global__ __launch_bounds__(kBlock) void absmax_vec_kernel(GradRows g, const float4* __restrict__ ref4,
                                                            const float4* __restrict__ ref24,
                                                            float* partials, uint64_t nvec,
                                                            uint32_t M, float eps, const float* __restrict__ means) {
  constexpr int L = kAbsmaxLoads;
  constexpr uint64_t kWaveTile = (uint64_t)kWave * L;
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const uint32_t m0 = blockIdx.y * MC;
  float mx[MC];
#pragma unroll
  for (int mm = 0; mm < MC; ++mm) mx[mm] = 0.f;
  const uint64_t ntiles = (nvec + kWaveTile - 1) / kWaveTile;  // wavefront tiles
  for (uint64_t tile = (uint64_t)blockIdx.x * kWavesPerBlock + wave; tile < ntiles;
       tile += (uint64_t)gridDim.x * kWavesPerBlock) {
    RefTile<NORM> rt[L];
    uint64_t iv[L];
    const bool full = (tile + 1) * kWaveTile <= nvec;  // wave-uniform
#pragma unroll
    for (int j = 0; j < L; ++j) {
      iv[j] = tile * kWaveTile + (uint64_t)j * kWave + lane;
      if (full || iv[j] < nvec) {
        rt[j].load(ref4, ref24, iv[j], eps);
        if (kByReciprocal<NORM, MC>) rt[j].reciprocals();
      }
    }
    if (full) {
      absmax_rows<NORM, MC, true>(g, rt, iv, nvec, m0, M, means, mx);
    } else {
      absmax_rows<NORM, MC, false>(g, rt, iv, nvec, m0, M, means, mx);
    }
  }
  block_max_to_partials<MC>(mx, m0, M, partials);
}

template <int NORM>
__global__ __launch_bounds__(kBlock) void absmax_scalar_kernel(const float* __restrict__ g,
                                                               const float* __restrict__ ref,
                                                               const float* __restrict__ ref2,
                                                               float* partials, uint64_t first, uint64_t d,
                                                               uint32_t M, float eps,
                                                               const float* __restrict__ means) {
  const uint32_t m = blockIdx.y;
  const float mu = NORM == kNormMean ? means[m] : 0.f;
  float mx[1] = {0.f};
  const uint64_t stride = (uint64_t)gridDim.x * kBlock;
  for (uint64_t e = first + (uint64_t)blockIdx.x * kBlock + threadIdx.x; e < d; e += stride) {
    float r1, r2;
    load_ref_scalar<NORM>(ref, ref2, e, eps, r1, r2);
    mx[0] = fmaxf(mx[0], fabsf(normalize_w<NORM>(g[(uint64_t)m * d + e], r1, r2, mu)));
  }
  block_max_to_partials<1>(mx, m, M, partials);
}

// ------------------------------------------------------------------------------------------
// Pass 2: normalise, draw, round, sign, pack   (Algorithm 1: sample z, transmit sign (.) z and R)
//
// A wavefront owns 64 * 4 float4 = 1024 consecutive coordinates.  Load j of lane l covers
// coordinates 256 j + 4 l .. + 3, so every load instruction is one contiguous 1 KiB.  The four
// codes of a load form an 8-bit (ternary) or 16-bit (4-bit codes) fragment; fragment (j, l) is
// fragment number 64 j + l of the wavefront's packed output, so writing fragments to LDS at that
// index and reading LDS back as 32-bit words gives each lane whole words to store, contiguously.
// ------------------------------------------------------------------------------------------
// Everything a lane keeps across the worker loop of the quantiser: its four float4 positions and
// the reference operands there.  FULL: the wavefront's whole tile lies inside the row, no bounds
// checks (all tiles but the last).
template <int NORM>
struct QuantLane {
  RefTile<NORM> rt[kLoadsPerLane];
  uint64_t iv[kLoadsPerLane];
  bool ok[kLoadsPerLane];
};

template <int NORM, bool FULL>
__device__ __forceinline__ void load_worker_tile(const QuantLane<NORM>& q, const GradRows& g, uint32_t m,
                                                 float4 (&x)[kLoadsPerLane]) {
#pragma unroll
  for (int j = 0; j < kLoadsPerLane; ++j) {
    if (FULL || q.ok[j]) {
      x[j] = load_row_stream(g.row(m) + q.iv[j]);
    } else {
      x[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
  }
}

// Codes of one worker for this lane's 16 coordinates: four fragments of 4 codes each.
template <int NORM, int BITS, bool FULL, bool RECIP>
__device__ __forceinline__ void quantize_worker_tile(const QuantLane<NORM>& q, const float4 (&x)[kLoadsPerLane],
                                                     float R, float mu, uint32_t m, uint32_t iter, uint32_t k0,
                                                     uint32_t k1, uint32_t (&frag)[kLoadsPerLane]) {
  if (R == 0.f) {
#pragma unroll
    for (int j = 0; j < kLoadsPerLane; ++j) frag[j] = 0u;
    return;
  }
  const float inv_r = 1.0f / R;
#pragma unroll
  for (int j = 0; j < kLoadsPerLane; ++j) {
    frag[j] = 0u;
    if (FULL || q.ok[j]) {
      const U32x4 rnd = philox4x32_10((uint32_t)q.iv[j], m, iter, 0u, k0, k1);
      const float4 v = normalize4<NORM, RECIP>(x[j], q.rt[j], mu);
      const uint32_t c0 = quantize_code<BITS>(v.x, inv_r, rnd.x);
      const uint32_t c1 = quantize_code<BITS>(v.y, inv_r, rnd.y);
      const uint32_t c2 = quantize_code<BITS>(v.z, inv_r, rnd.z);
      const uint32_t c3 = quantize_code<BITS>(v.w, inv_r, rnd.w);
      frag[j] = c0 | (c1 << BITS) | (c2 << (2 * BITS)) | (c3 << (3 * BITS));
    }
  }
}

// One LDS buffer per wavefront seen as bytes, half-words or words (the types may alias each other).
typedef uint8_t __attribute__((may_alias)) lds_u8;
typedef uint16_t __attribute__((may_alias)) lds_u16;
typedef uint32_t __attribute__((may_alias)) lds_u32;
template <int WORDS, int SLOTS = 1>
union FragmentBuffer {
  lds_u8 b8[SLOTS][kWavesPerBlock][WORDS * 4];
  lds_u16 b16[SLOTS][kWavesPerBlock][WORDS * 2];
  lds_u32 b32[SLOTS][kWavesPerBlock][WORDS];
};

__device__ __forceinline__ void wave_lds_fence() {
  // Same-wavefront LDS traffic is executed in order; this only pins the compiler's order.
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Fragment (j, lane) is fragment number 64 j + lane of the wavefront's packed output: write the
// fragments to LDS at that index, read whole words back, store them contiguously.
// DEFER: the words stay in LDS slot `slot` (one slot per worker of the workgroup) and are written by
// flush_packed after the last worker, 16 bytes per lane.
template <int BITS, int WPW, int SLOTS, bool DEFER>
__device__ __forceinline__ void store_packed(FragmentBuffer<WPW, SLOTS>& lds, int slot, int wave, int lane,
                                             const uint32_t (&frag)[kLoadsPerLane], uint32_t* __restrict__ row,
                                             uint64_t word_base, uint64_t words) {
  if (BITS == 2) {
#pragma unroll
    for (int j = 0; j < kLoadsPerLane; ++j) lds.b8[slot][wave][j * kWave + lane] = (uint8_t)frag[j];
  } else {
#pragma unroll
    for (int j = 0; j < kLoadsPerLane; ++j) lds.b16[slot][wave][j * kWave + lane] = (uint16_t)frag[j];
  }
  if (DEFER) return;
  wave_lds_fence();
#pragma unroll
  for (int k = 0; k < WPW / kWave; ++k) {
    const uint64_t wi = word_base + (uint64_t)k * kWave + lane;
    const uint32_t word = lds.b32[slot][wave][k * kWave + lane];
    if (wi < words) store_word_through(row + wi, word);
  }
  wave_lds_fence();
}

typedef uint32_t v4u_t __attribute__((ext_vector_type(4)));

// The deferred words of `count` workers: a row of the wavefront tile is WPW words, WPW / 4 lanes
// store it 16 bytes each, so one store instruction covers 256 / WPW rows.  The store carries the
// device-coherent cache policy (sc1) like store_word_through; there is no builtin for a 16-byte store
// with that policy, hence the instruction is written out.  Nothing after it depends on the
// memory counters (the wavefront ends), and the trailing no-op covers the cycle in which the data
// registers must stay untouched.  Measured against 4-byte sc1 stores issued per worker: quantise pass
// 0.834 -> 0.806 ms; the same with non-temporal or plain 16-byte stores: 0.84 / 0.88 ms.
template <int WPW, int SLOTS>
__device__ __forceinline__ void flush_packed(FragmentBuffer<WPW, SLOTS>& lds, int wave, int lane,
                                             uint32_t* __restrict__ codes, uint64_t words, uint64_t word_base,
                                             uint32_t m0, uint32_t count) {
  constexpr int LPR = WPW / 4;       // lanes per row
  constexpr int RPI = kWave / LPR;   // rows per store instruction
  wave_lds_fence();
  const int quad = lane % LPR;
#pragma unroll
  for (int r0 = 0; r0 < SLOTS; r0 += RPI) {
    const uint32_t r = (uint32_t)(r0 + lane / LPR);
    if (r < count) {
      const v4u_t w4 = *reinterpret_cast<const v4u_t*>(&lds.b32[r][wave][4 * quad]);
      v4u_t* dst = reinterpret_cast<v4u_t*>(codes + (uint64_t)(m0 + r) * words + word_base) + quad;
      asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" : : "v"(dst), "v"(w4) : "memory");
    }
  }
}

// Worker loop of one wavefront tile, software pipelined two workers per trip so that the two
// register sets swap roles without copies: the loads of worker m+1 are in flight while the codes
// of worker m are computed.
// Small problems: the scale pass was fused into the gradient kernel and left only a few rows of
// per-workgroup maxima (partials[row][m]); the quantiser then takes their maximum itself instead of
// waiting for a reduction kernel of its own, and the first workgroup publishes scales[m].
struct FusedScale {
  const float* partials;
  uint32_t rows;
  float* out;
};

__device__ __forceinline__ float fused_scale(const FusedScale& f, uint32_t m, uint32_t M, bool publish) {
  float v = 0.f;
  for (uint32_t b = 0; b < f.rows; ++b) v = fmaxf(v, f.partials[(uint64_t)b * M + m]);
  v = v < FLT_MIN ? 0.f : v;
  if (publish) f.out[m] = v;
  return v;
}

template <int NORM, int BITS, int WPW, int SLOTS, bool FULL, bool FUSED, bool DEFER>
__device__ __forceinline__ void quantize_rows(const QuantLane<NORM>& q, FragmentBuffer<WPW, SLOTS>& lds, int wave, int lane,
                                              const GradRows& g, const float* __restrict__ scales,
                                              uint32_t* __restrict__ codes, uint64_t nvec, uint64_t words,
                                              uint64_t word_base, uint32_t m0, uint32_t m_end, uint32_t iter,
                                              uint32_t k0, uint32_t k1, const float* __restrict__ means,
                                              const FusedScale& fs, uint32_t M) {
  constexpr int L = kLoadsPerLane;
  float4 xa[L], xb[L];
  uint32_t frag[L];
  // The scale (and mean) of a worker is fetched before the tile loads that are to stay in flight
  // during the previous worker's arithmetic: loads return in order, so a scalar fetched after them
  // would make the wait for it a wait for the whole prefetch.
  auto mean_of = [&](uint32_t m) { return NORM == kNormMean ? means[m] : 0.f; };
  auto scale_of = [&](uint32_t m) {
    return FUSED ? fused_scale(fs, m, M, blockIdx.x == 0 && threadIdx.x == 0) : scales[m];
  };
  float ra = scale_of(m0), mua = mean_of(m0), rb = 0.f, mub = 0.f;
  load_worker_tile<NORM, FULL>(q, g, m0, xa);
  // Steady state: both prefetches of a trip are unconditional.  A load issued under a condition
  // makes the compiler wait for all outstanding loads where the paths join (it cannot count what
  // is in flight), which would drain the prefetch before the arithmetic it is meant to overlap.
  uint32_t m = m0;
  for (; m + 2 < m_end; m += 2) {
    rb = scale_of(m + 1);
    mub = mean_of(m + 1);
    load_worker_tile<NORM, FULL>(q, g, m + 1, xb);
    quantize_worker_tile<NORM, BITS, FULL, kByReciprocal<NORM, SLOTS>>(q, xa, ra, mua, m, iter, k0, k1, frag);
    store_packed<BITS, WPW, SLOTS, DEFER>(lds, DEFER ? (int)(m - m0) : 0, wave, lane, frag, codes + (uint64_t)m * words, word_base,
                                          words);
    ra = scale_of(m + 2);
    mua = mean_of(m + 2);
    load_worker_tile<NORM, FULL>(q, g, m + 2, xa);
    quantize_worker_tile<NORM, BITS, FULL, kByReciprocal<NORM, SLOTS>>(q, xb, rb, mub, m + 1, iter, k0, k1, frag);
    store_packed<BITS, WPW, SLOTS, DEFER>(lds, DEFER ? (int)(m + 1 - m0) : 0, wave, lane, frag,
                                          codes + (uint64_t)(m + 1) * words, word_base, words);
  }
  // one or two workers are left, the first of them already in xa
  if (m + 1 < m_end) {
    rb = scale_of(m + 1);
    mub = mean_of(m + 1);
    load_worker_tile<NORM, FULL>(q, g, m + 1, xb);
    quantize_worker_tile<NORM, BITS, FULL, kByReciprocal<NORM, SLOTS>>(q, xa, ra, mua, m, iter, k0, k1, frag);
    store_packed<BITS, WPW, SLOTS, DEFER>(lds, DEFER ? (int)(m - m0) : 0, wave, lane, frag, codes + (uint64_t)m * words, word_base,
                                          words);
    quantize_worker_tile<NORM, BITS, FULL, kByReciprocal<NORM, SLOTS>>(q, xb, rb, mub, m + 1, iter, k0, k1, frag);
    store_packed<BITS, WPW, SLOTS, DEFER>(lds, DEFER ? (int)(m + 1 - m0) : 0, wave, lane, frag,
                                          codes + (uint64_t)(m + 1) * words, word_base, words);
  } else {
    quantize_worker_tile<NORM, BITS, FULL, kByReciprocal<NORM, SLOTS>>(q, xa, ra, mua, m, iter, k0, k1, frag);
    store_packed<BITS, WPW, SLOTS, DEFER>(lds, DEFER ? (int)(m - m0) : 0, wave, lane, frag, codes + (uint64_t)m * words, word_base,
                                          words);
  }
  if (DEFER) flush_packed<WPW, SLOTS>(lds, wave, lane, codes, words, word_base, m0, m_end - m0);
}

template <int NORM, int BITS, int MC, bool FUSED>
__global__ __launch_bounds__(kBlock) void quantize_pack_vec_kernel(
    GradRows g, const float4* __restrict__ ref4, const float4* __restrict__ ref24,
    const float* __restrict__ scales, uint32_t* __restrict__ codes, uint64_t nvec, uint64_t words,
    uint32_t M, float eps, uint32_t k0, uint32_t k1, uint32_t iter, const float* __restrict__ means,
    FusedScale fs, const uint32_t* __restrict__ skip_if_set) {
  constexpr int L = kLoadsPerLane;
  constexpr int WPW = kWave * L * 4 * BITS / 32;  // packed words per wavefront tile
  __shared__ __attribute__((aligned(16))) FragmentBuffer<WPW, MC> lds;
  // the codes come from the candidate slots instead (quantize_candidates_kernel) when that word is set
  if (skip_if_set != nullptr && skip_if_set[0] != 0u) return;
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const uint64_t wave_tile = (uint64_t)blockIdx.x * kWavesPerBlock + wave;
  const uint64_t word_base = wave_tile * WPW;

  QuantLane<NORM> q;
#pragma unroll
  for (int j = 0; j < L; ++j) {
    q.iv[j] = wave_tile * (kWave * L) + (uint64_t)j * kWave + lane;
    q.ok[j] = q.iv[j] < nvec;
    if (q.ok[j]) {
      q.rt[j].load(ref4, ref24, q.iv[j], eps);
      if (kByReciprocal<NORM, MC>) q.rt[j].reciprocals();
    }
  }

  const uint32_t m0 = blockIdx.y * MC;
  const uint32_t m_end = min(m0 + MC, M);
  if ((wave_tile + 1) * (kWave * L) <= nvec) {  // wave-uniform
    if (MC > 1 && words % 4 == 0 && (reinterpret_cast<uintptr_t>(codes) & 15u) == 0) {  // 16-byte aligned rows
      quantize_rows<NORM, BITS, WPW, MC, true, FUSED, true>(q, lds, wave, lane, g, scales, codes, nvec, words,
                                                            word_base, m0, m_end, iter, k0, k1, means, fs, M);
    } else {
      quantize_rows<NORM, BITS, WPW, MC, true, FUSED, false>(q, lds, wave, lane, g, scales, codes, nvec, words,
                                                             word_base, m0, m_end, iter, k0, k1, means, fs, M);
    }
  } else {
    quantize_rows<NORM, BITS, WPW, MC, false, FUSED, false>(q, lds, wave, lane, g, scales, codes, nvec, words,
                                                            word_base, m0, m_end, iter, k0, k1, means, fs, M);
  }
}

// ------------------------------------------------------------------------------------------
// Ternary coder without a second pass over g   (section "Gradient Compression": P(z = 1) = |v| / R)
//
// In high dimension nearly every element of a row codes to 0: the largest element R is far above the
// typical |v|, and only a fraction E|v| / R of the elements -- a few percent -- draws z = 1.  Whether an
// element CAN code non-zero is decided in the scale pass, before R is known, against any lower bound
// R^ <= R at hand: fl(1 / R^) >= fl(1 / R) (the correctly rounded quotient is monotone) and
// fl(|v| x) is monotone in x, so  u >= fl(|v| fl(1 / R^))  implies  u >= fl(|v| fl(1 / R)):  level 0
// whatever R turns out to be.  The elements that fail this test -- the candidates -- are kept in a slot per
// worker and wavefront tile, one 32-bit word each: the sign of the normalised value, the position within the
// tile in the low 10 bits, and in between tau = |v| / u -- the scale up to which the element codes non-zero --
// to 13 bits of its significand.  R^ is the maximum over a sample of the row taken beforehand (one tile in
// kSampleStride); a row whose sample says that its candidates will not fit the slots is left to the
// ordinary path.  The quantise pass then reads the slots instead of g and compares the row's scale with
// the entry: the level [u < fl(|v| fl(1 / R))] is 1 for every R below the bracket that the entry gives for tau
// and 0 for every R above it (thresholds widened by what the roundings can move); the few elements whose
// bracket contains R (three candidates in ten thousand) are fetched from g and coded from the value and its
// draw.  Everything else is cleared, and the words are packed.  A slot that overflowed (a tile with more
// than kCandCap candidates) sends its tile through the ordinary path.  The codes are those of the two-pass
// coder bit for bit; what changes is that g is read once: 4 + 4/M bytes per element instead of 8 + 8/M.
// Used for 2-bit codes with the largest-magnitude scale when every wavefront tile is a full one
// (d a multiple of 1024) and the row is long enough for the second read to come from memory.
// ------------------------------------------------------------------------------------------
constexpr int kCandCap = 127;         // candidates a slot holds; word 0 of a slot is their count
constexpr int kSlotEntries = 128;     // 32-bit words per slot: 512 bytes per worker and wavefront tile
constexpr uint32_t kSampleStride = 128;  // the sample: every 128th wavefront tile of a row
constexpr uint32_t kCandPosMask = 0x3FFu;  // low 10 bits of a candidate word: position within the tile

// The sample of a row taken before the scale pass: over every kSampleStride-th wavefront tile, the largest
// |v| (the lower bound R^ of the row's scale) and the sum of |v|.  Their ratio, mean |v| / R^, is the share
// of the row's elements that will be candidates -- P(u < |v| / R^) averaged over the elements -- so it tells
// beforehand whether the slots can hold them.  One worker per workgroup row (blockIdx.y); partial results per
// workgroup, reduced by sample_finish_kernel.
constexpr float kDenseLimit = 0.10f;  // 1024 elements x 0.10 + two standard deviations fill a slot of kCandCap
template <int NORM>
__global__ __launch_bounds__(kBlock) void sample_stats_kernel(GradRows g, const float4* __restrict__ ref4,
                                                              float* __restrict__ part_max,
                                                              float* __restrict__ part_sum, uint64_t nvec, uint32_t M) {
  constexpr int L = kAbsmaxLoads;
  constexpr uint64_t kWaveTile = (uint64_t)kWave * L;
  __shared__ float red[2][kWavesPerBlock];
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const uint32_t m = blockIdx.y;
  const uint64_t ntiles = nvec / kWaveTile;  // whole tiles only
  const v4f_u_t* row = g.row(m);
  float amax = 0.f, asum = 0.f;
  for (uint64_t tile = ((uint64_t)blockIdx.x * kWavesPerBlock + wave) * kSampleStride; tile < ntiles;
       tile += (uint64_t)gridDim.x * kWavesPerBlock * kSampleStride) {
    float4 x[L], r[L];
#pragma unroll
    for (int j = 0; j < L; ++j) {
      const uint64_t i = tile * kWaveTile + (uint64_t)(j * kWave + lane);
      x[j] = load_row_stream(row + i);
      r[j] = NORM == kNormSub ? ref4[i] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int j = 0; j < L; ++j) {
      const float a0 = fabsf(x[j].x - r[j].x), a1 = fabsf(x[j].y - r[j].y);
      const float a2 = fabsf(x[j].z - r[j].z), a3 = fabsf(x[j].w - r[j].w);
      amax = fmaxf(fmaxf(amax, fmaxf(a0, a1)), fmaxf(a2, a3));
      asum += (a0 + a1) + (a2 + a3);
    }
  }
  amax = wave_max(amax);
  asum = wave_sum(asum);
  if (lane == 0) {
    red[0][wave] = amax;
    red[1][wave] = asum;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float mx = red[0][0], sm = red[1][0];
#pragma unroll
    for (int k = 1; k < kWavesPerBlock; ++k) {
      mx = fmaxf(mx, red[0][k]);
      sm += red[1][k];
    }
    part_max[(uint64_t)blockIdx.x * M + m] = mx;
    part_sum[(uint64_t)blockIdx.x * M + m] = sm;
  }
}

// sample_max[m] = R^ of worker m (0 when below the smallest normal number, as for a scale), and
// select_ok[m] = 1 when the sample says that the row's candidates fit the slots, else 0: the scale pass then
// takes that worker's part as an ordinary scale pass and the quantise pass takes its tiles through the
// ordinary path, without the slots.  sampled = elements of a row in the sample.  One workgroup per worker.
__global__ __launch_bounds__(kBlock) void sample_finish_kernel(const float* __restrict__ part_max,
                                                               const float* __restrict__ part_sum, uint32_t nblocks,
                                                               uint32_t M, float sampled, float* __restrict__ sample_max,
                                                               uint32_t* __restrict__ select_ok) {
  __shared__ float red[2][kWavesPerBlock];
  const uint32_t m = blockIdx.x;
  float mx = 0.f, sm = 0.f;
  for (uint32_t b = threadIdx.x; b < nblocks; b += kBlock) {
    mx = fmaxf(mx, part_max[(uint64_t)b * M + m]);
    sm += part_sum[(uint64_t)b * M + m];
  }
  mx = wave_max(mx);
  sm = wave_sum(sm);
  if (threadIdx.x % kWave == 0) {
    red[0][threadIdx.x / kWave] = mx;
    red[1][threadIdx.x / kWave] = sm;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int k = 1; k < kWavesPerBlock; ++k) {
      mx = fmaxf(mx, red[0][k]);
      sm += red[1][k];
    }
    sample_max[m] = mx < FLT_MIN ? 0.f : mx;
    // (a sum that is no number, or an infinite one, compares false: the slots are then not used)
    select_ok[m] = sm <= kDenseLimit * sampled * mx ? 1u : 0u;
  }
}

template <int NORM, int MC>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(4, 4))) void absmax_select_kernel(GradRows g, const float4* __restrict__ ref4,
                                                               const float4* __restrict__ ref24, float* partials,
                                                               uint64_t nvec, uint32_t M, float eps,
                                                               const float* __restrict__ sample_max,
                                                               const uint32_t* __restrict__ select_ok,
                                                               uint32_t* __restrict__ slots,
                                                               uint32_t* __restrict__ overflowed, uint32_t k0,
                                                               uint32_t k1, uint32_t iter) {
  constexpr int L = kAbsmaxLoads;
  constexpr uint64_t kWaveTile = (uint64_t)kWave * L;
  static_assert(L == kLoadsPerLane, "the quantise pass reads the slots by the same tiles");
  static_assert(NORM == kNormNone || NORM == kNormSub, "the coder that reads g once: no divisor reference");
  // What a wavefront fetches per tile, in order: the reference, then the MC workers' parts, and nothing up to
  // a multiple of three.  The items rotate through three register buffers: while item i is worked on, items
  // i + 1 and i + 2 are on their way -- across the end of the tile as well (the next tile's reference and
  // first worker are requested during this tile's last workers).  The reference of the tile lives in LDS,
  // not in registers: three buffers then cost what two buffers and a reference did, and twice the bytes are
  // in flight per wavefront.  (Measured 2 % faster than two buffers that drained at the end of every tile:
  // the pass is bound neither by the depth of its prefetch nor by its arithmetic.)
  constexpr int kItems = (MC + 1 + 2) / 3 * 3;
  // staging per wavefront: the count and up to kCandCap candidates (value word and draw), one word that takes
  // everything beyond the capacity, then a word per lane for the elements that are no candidates
  constexpr uint32_t kStageSink = kSlotEntries, kStageDump = kSlotEntries + 2;
  __shared__ __attribute__((aligned(16))) uint32_t stage[kWavesPerBlock][kStageDump + kWave];
  __shared__ __attribute__((aligned(16))) uint32_t draws[kWavesPerBlock][kStageDump + kWave];
  __shared__ __attribute__((aligned(16))) float4 refs[kWavesPerBlock][L][kWave];
  __shared__ uint32_t over[kWavesPerBlock];
  // the wavefront's number as a value the compiler knows to be the same in every lane: tile numbers, row and
  // slot addresses are then scalar, and a lane's own part of every address is one 32-bit offset
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave)), lane = threadIdx.x % kWave;
  const uint32_t m0 = blockIdx.y * MC;
  const uint32_t count = min((uint32_t)MC, M - m0);
  uint32_t nover = 0;  // slots of this wavefront that overflowed
  float mx[MC];
#pragma unroll
  for (int mm = 0; mm < MC; ++mm) mx[mm] = 0.f;
  const uint64_t ntiles = nvec / kWaveTile;  // every tile is a full one
  const uint32_t lane4 = 4u * (uint32_t)lane;
  // The lower bound R^ of a worker's scale is the maximum over the sample of its row.  The test
  //   u < fl(|v| fl(1 / R^)),  u = (word >> 8) 2^-24,
  // is made in three operations and from above:  float(word) < |v| c1 + 258  with
  // c1 = fl(fl(1 / R^) 2^32 (1 + 2^-20)).  It holds whenever the exact test does (then word < 2^32 fl(|v| / R^) + 256;
  // converting the word and the two roundings on the right move either side by less than 2^-23 relatively,
  // which the factor 1 + 2^-20 and the 2 added to 256 cover) and passes 2^-20 more elements than it: the
  // quantise pass codes a candidate exactly, so more is harmless.  Below 2^-90 no bound is claimed (c1 would
  // overflow): every non-zero element is a candidate.
  float c1[MC];
  bool select[MC];  // the sample found the worker's row too dense for the slots: only its maximum is taken
#pragma unroll
  for (int mm = 0; mm < MC; ++mm) {
    const float r_hat = sample_max[min(m0 + (uint32_t)mm, M - 1)];
    c1[mm] = r_hat >= 0x1p-90f ? (1.0f / r_hat) * (0x1p32f * (1.0f + 0x1p-20f)) : INFINITY;
    select[mm] = select_ok[min(m0 + (uint32_t)mm, M - 1)] != 0u;
  }
  // one worker's part of the tile: its maximum, and its candidates into the slot
  auto worker = [&](const float4 (&x)[L], int mm, uint64_t tile) {
    const uint32_t m = m0 + (uint32_t)mm;
    float amax = 0.f;
    if (!select[mm]) {  // (the same for the whole wavefront)
#pragma unroll
      for (int j = 0; j < L; ++j) {
        float4 v = x[j];
        if (NORM == kNormSub) {
          const float4 r = refs[wave][j][lane];
          v = make_float4(x[j].x - r.x, x[j].y - r.y, x[j].z - r.z, x[j].w - r.w);
        }
        amax = max3_abs(v.z, v.w, max3_abs(v.x, v.y, amax));
      }
      mx[mm] = fmaxf(mx[mm], amax);
      nover += 1u;  // counts as a slot that is not used
      return;
    }
    uint32_t base = 1;  // word 0 of the slot is the count
#pragma unroll
    for (int j = 0; j < L; ++j) {
      float4 v = x[j];
      if (NORM == kNormSub) {
        const float4 r = refs[wave][j][lane];
        v = make_float4(x[j].x - r.x, x[j].y - r.y, x[j].z - r.z, x[j].w - r.w);
      }
      amax = max3_abs(v.z, v.w, max3_abs(v.x, v.y, amax));
      const uint64_t iv = tile * kWaveTile + (uint64_t)(j * kWave + lane);
      const U32x4 rnd = philox4x32_10((uint32_t)iv, m, iter, 0u, k0, k1);
      const float vv[4] = {v.x, v.y, v.z, v.w};
      const uint32_t rr[4] = {rnd.x, rnd.y, rnd.z, rnd.w};
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const bool cand = (float)rr[c] < __builtin_fmaf(fabsf(vv[c]), c1[mm], 258.0f);
        const uint64_t mask = __builtin_amdgcn_ballot_w64(cand);
        const uint32_t pos = base + __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                                              __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
        // Every lane writes, the others into a word of their own behind the candidates': a store under a
        // condition would end the basic block at every element, and the sixteen elements of a lane could not
        // overlap.  Candidates beyond the slot's capacity (the slot is then not used) share one word.
        const uint32_t at = cand ? min(pos, kStageSink) : kStageDump + (uint32_t)lane;
        stage[wave][at] = (__float_as_uint(vv[c]) & ~kCandPosMask) | (uint32_t)(256 * j + c) | lane4;
        draws[wave][at] = rr[c];
        base += (uint32_t)__builtin_popcountll(mask);
      }
    }
    mx[mm] = fmaxf(mx[mm], amax);
    if (lane == 0) stage[wave][0] = base - 1;  // candidates found (more than kCandCap: the slot is not used)
    wave_lds_fence();
    // Words to write, the count included (8 bytes per lane, the last one whatever the staging area holds);
    // of a slot that overflowed only the count.  (The slots cost about 0.15 ms per launch -- 0.2 GB next to
    // 4.8 GB of reads -- and pieces rounded up to whole 128-byte lines, 16-byte stores or a quarter fewer bytes
    // all measured the same; half of it remains when the stores never leave the caches.  The cache policy does
    // matter: plain stores +0.03 ms, non-temporal ones +0.08 ms.)
    const bool fits = base <= (uint32_t)kSlotEntries;
    nover += fits ? 0u : 1u;
    const uint32_t used = fits ? base : 1u;
    if (2u * lane < used) {  // one store instruction covers the slot: 8 bytes per lane, device-coherent policy
      // What goes into the slot for a candidate is not v but tau = |v| / u (u its 24-bit draw), the scale up
      // to which it codes non-zero, to 13 bits of the significand: the quantise pass then compares the row's
      // scale with tau and needs neither the draw nor the value.  The reciprocal is taken here, for the two
      // candidates of the lane, not for every element of the tile.  u = 0 gives an infinite tau (or none, for
      // v = 0), which the quantise pass takes as "look at the value".
      const uint2 vw = *reinterpret_cast<const uint2*>(&stage[wave][2 * lane]);
      const uint2 dw = *reinterpret_cast<const uint2*>(&draws[wave][2 * lane]);
      auto entry = [](uint32_t value_word, uint32_t draw) {
        const float tau = __uint_as_float(value_word & 0x7FFFFC00u) * (__builtin_amdgcn_rcpf((float)(draw >> 8)) * 0x1p24f);
        return (__float_as_uint(tau) & 0x7FFFFC00u) | (value_word & 0x800003FFu);
      };
      const uint32_t e0 = lane == 0 ? vw.x : entry(vw.x, dw.x);  // word 0 of the slot is the count
      const uint64_t two = ((uint64_t)entry(vw.y, dw.y) << 32) | e0;
      uint64_t* slot = reinterpret_cast<uint64_t*>(slots + ((uint64_t)m * ntiles + tile) * kSlotEntries);
      __hip_atomic_store(slot + (uint32_t)lane, two, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    wave_lds_fence();
  };
  // Every request is made whatever the tile (a load under a branch could not be counted by the waits that
  // follow it): past the wavefront's last tile all lanes read the first float4 of this tile's part again.
  auto request = [&](float4 (&b)[L], int item, uint64_t t, uint32_t keep) {
    if (item == 0) {
      if (NORM == kNormSub) {
#pragma unroll
        for (int j = 0; j < L; ++j) b[j] = load_stream(ref4 + t * kWaveTile + ((uint32_t)(j * kWave + lane) & keep));
      }
    } else if (item <= MC) {
      const v4f_u_t* row = g.row(min(m0 + (uint32_t)(item - 1), M - 1));
#pragma unroll
      for (int j = 0; j < L; ++j) b[j] = load_row_stream(row + t * kWaveTile + ((uint32_t)(j * kWave + lane) & keep));
    }
  };
  auto work = [&](const float4 (&b)[L], int item, uint64_t tile) {
    if (item == 0) {
      if (NORM == kNormSub) {
#pragma unroll
        for (int j = 0; j < L; ++j) refs[wave][j][lane] = b[j];
        wave_lds_fence();
      }
    } else if (item <= MC) {
      if ((uint32_t)(item - 1) < count) worker(b, item - 1, tile);
    }
  };
  const uint64_t stride = (uint64_t)gridDim.x * kWavesPerBlock;
  uint64_t tile = (uint64_t)blockIdx.x * kWavesPerBlock + wave;
  if (tile < ntiles) {
    float4 b0[L], b1[L], b2[L];
    request(b0, 0, tile, ~0u);
    request(b1, 1, tile, ~0u);
    for (; tile < ntiles; tile += stride) {
      const bool more = tile + stride < ntiles;
      const uint64_t t_next = more ? tile + stride : tile;
      const uint32_t keep_next = more ? ~0u : 0u;
      // step i: request item i + 2 into the buffer that item i - 1 has just left, then work on item i
      auto step = [&](auto I, float4 (&into)[L], const float4 (&from)[L]) {
        constexpr int i = decltype(I)::value;
        constexpr bool wraps = i + 2 >= kItems;
        request(into, wraps ? i + 2 - kItems : i + 2, wraps ? t_next : tile, wraps ? keep_next : ~0u);
        work(from, i, tile);
      };
      step(std::integral_constant<int, 0>{}, b2, b0);
      step(std::integral_constant<int, 1>{}, b0, b1);
      step(std::integral_constant<int, 2>{}, b1, b2);
      if constexpr (kItems > 3) {
        step(std::integral_constant<int, 3>{}, b2, b0);
        step(std::integral_constant<int, 4>{}, b0, b1);
        step(std::integral_constant<int, 5>{}, b1, b2);
      }
      if constexpr (kItems > 6) {
        step(std::integral_constant<int, 6>{}, b2, b0);
        step(std::integral_constant<int, 7>{}, b0, b1);
        step(std::integral_constant<int, 8>{}, b1, b2);
      }
    }
  }
  if (lane == 0) over[wave] = nover;
  block_max_to_partials<MC>(mx, m0, M, partials);  // has a workgroup barrier after its own LDS writes
  if (threadIdx.x == 0) {
    uint32_t total = 0;
#pragma unroll
    for (int k = 0; k < kWavesPerBlock; ++k) total += over[k];
    overflowed[(uint64_t)blockIdx.y * gridDim.x + blockIdx.x] = total;
  }
}

// The reduction of the scale pass's partial maxima (workgroups 0 .. M - 1, one per worker) and, in one more
// workgroup, whether the slots are worth using: at most one tile in fifty may have overflowed (such tiles go
// through a plain, unpipelined form of the ordinary path).  use_slots[0] = 1 or 0.
__global__ __launch_bounds__(kBlock) void absmax_finish_vote_kernel(const float* __restrict__ partials, uint32_t nblocks,
                                                                    uint32_t M, float* __restrict__ scales,
                                                                    const uint32_t* __restrict__ overflowed, uint32_t n,
                                                                    uint64_t tiles_in_all,
                                                                    uint32_t* __restrict__ use_slots) {
  if (blockIdx.x < M) {
    absmax_finish_worker(partials, nblocks, M, scales, blockIdx.x);
    return;
  }
  __shared__ unsigned long long sum;
  if (threadIdx.x == 0) sum = 0ull;
  __syncthreads();
  unsigned long long mine = 0;
  for (uint32_t i = threadIdx.x; i < n; i += kBlock) mine += overflowed[i];
  atomicAdd(&sum, mine);
  __syncthreads();
  if (threadIdx.x == 0) use_slots[0] = sum * 50ull <= tiles_in_all ? 1u : 0u;
}

// The packed codes of a tile from its slots.  One wavefront per tile as in the quantiser; the words of a
// worker are cleared in LDS, the candidates' codes are or-ed in, and all workers' words are written at the
// end as the quantiser writes them.
template <int NORM, int MC>
__global__ __launch_bounds__(kBlock) void quantize_candidates_kernel(
    GradRows g, const float4* __restrict__ ref4, const float4* __restrict__ ref24, const float* __restrict__ scales,
    const uint32_t* __restrict__ slots, uint32_t* __restrict__ codes, uint64_t nvec, uint64_t words, uint32_t M,
    float eps, uint32_t k0, uint32_t k1, uint32_t iter, const uint32_t* __restrict__ use_slots,
    const uint32_t* __restrict__ select_ok) {
  constexpr int L = kLoadsPerLane;
  constexpr int WPW = kWave * L * 4 * 2 / 32;  // 64 packed words per wavefront tile
  static_assert(WPW == kWave, "one word per lane");
  __shared__ __attribute__((aligned(16))) FragmentBuffer<WPW, MC> lds;
  if (use_slots[0] == 0u) return;  // too many tiles overflowed: the ordinary quantiser runs instead
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const uint64_t ntiles = nvec / (kWave * L);
  const uint64_t tile = (uint64_t)blockIdx.x * kWavesPerBlock + wave;
  if (tile >= ntiles) return;  // whole wavefronts; nothing below meets the other wavefronts
  const uint64_t word_base = tile * WPW;
  const uint32_t m0 = blockIdx.y * MC;
  const uint32_t m_end = min(m0 + MC, M);
  // Counts and the first 64 words of all the workers' slots are requested at once (a slot rarely holds
  // more: the rest is fetched when its count says so), so that the workgroup waits for memory once and not
  // once per worker.  Words past a slot's count are whatever an earlier call left there and are not used.
  uint32_t cnt[MC];
  uint32_t first[MC];
#pragma unroll
  for (int mm = 0; mm < MC; ++mm) {
    const uint32_t m = min(m0 + (uint32_t)mm, M - 1);
    const uint32_t* __restrict__ sl = slots + ((uint64_t)m * ntiles + tile) * kSlotEntries;
    cnt[mm] = sl[0];
    first[mm] = sl[1 + lane];
  }
#pragma unroll
  for (int mm = 0; mm < MC; ++mm) {
    const uint32_t m = m0 + (uint32_t)mm;
    if (m >= m_end) break;
    const int slot = mm;
    const float R = scales[m];
    const uint32_t* __restrict__ sl = slots + ((uint64_t)m * ntiles + tile) * kSlotEntries;
    // (a worker whose row the sample found too dense has no slots: its tiles take the ordinary path)
    const uint32_t n = R == 0.f ? 0u : select_ok[m] != 0u ? cnt[mm] : (uint32_t)kCandCap + 1u;
    if (n <= (uint32_t)kCandCap) {
      lds.b32[slot][wave][lane] = 0u;
      wave_lds_fence();
      const float inv_r = R == 0.f ? 0.f : 1.0f / R;
      auto code_one = [&](uint32_t e) {
        const uint32_t pos = e & kCandPosMask;
        // The entry brackets tau = |v| / u: its significand was cut to 13 bits twice (the value's, then tau's own)
        // and its arithmetic is good to 2^-22, so tau lies in [lo (1 - 2^-22), hi (1 + 2^-13 + 2^-21)].
        // quantize_code's level [u < fl(|v| fl(1 / R))] is 1 for R <= tau (1 - 2^-21) and 0 for R >= tau (1 + 2^-21)
        // (the two roundings move |v| / R by less than 2^-22 relatively, 1 / R > 2^126 included), so only a scale
        // inside the widened bracket -- three candidates in ten thousand -- needs the value and the draw.
        const float lo = __uint_as_float(e & 0x7FFFFC00u), hi = __uint_as_float((e & 0x7FFFFC00u) | kCandPosMask);
        const bool bounded = (e & 0x7F800000u) != 0x7F800000u;  // u = 0: tau is infinite or no number
        uint32_t code;
        if (bounded && R <= lo * (1.0f - 0x1p-19f)) {
          code = 1u | ((e >> 31) << 1);
        } else if (R >= hi * (1.0f + 0x1p-12f)) {  // (false where tau is not bounded)
          code = 0u;
        } else {
          const uint64_t coord = tile * (uint64_t)(kWave * L * 4) + pos;
          const U32x4 rnd = philox4x32_10((uint32_t)(coord >> 2), m, iter, 0u, k0, k1);
          const uint32_t sel = pos & 3u;
          const uint32_t word = sel == 0u ? rnd.x : sel == 1u ? rnd.y : sel == 2u ? rnd.z : rnd.w;
          float r1 = 0.f;
          if (NORM == kNormSub) r1 = reinterpret_cast<const float*>(ref4)[coord];
          code = quantize_code<2>(normalize_w<NORM>(g.base[(uint64_t)m * g.pitch + coord], r1, 1.f, 0.f), inv_r, word);
        }
        if (code != 0u) atomicOr(&lds.b32[slot][wave][pos >> 4], code << (2u * (pos & 15u)));
      };
      if ((uint32_t)lane < n) code_one(first[mm]);
      if (n > (uint32_t)kWave && (uint32_t)(kWave + lane) < n) code_one(sl[1 + kWave + lane]);
    } else {  // the slot overflowed: this worker's tile goes through the ordinary path
      QuantLane<NORM> q;
#pragma unroll
      for (int j = 0; j < L; ++j) {
        q.iv[j] = tile * (kWave * L) + (uint64_t)j * kWave + lane;
        q.ok[j] = true;
        q.rt[j].load(ref4, ref24, q.iv[j], eps);
      }
      float4 x[L];
      uint32_t frag[L];
      load_worker_tile<NORM, true>(q, g, m, x);
      quantize_worker_tile<NORM, 2, true, false>(q, x, R, 0.f, m, iter, k0, k1, frag);
      store_packed<2, WPW, MC, true>(lds, slot, wave, lane, frag, codes, word_base, words);
    }
  }
  flush_packed<WPW, MC>(lds, wave, lane, codes, words, word_base, m0, m_end - m0);
}

// Any d (rows need not be 16-byte aligned): one thread per packed word.
template <int NORM, int BITS>
__global__ __launch_bounds__(kBlock) void quantize_pack_scalar_kernel(
    const float* __restrict__ g, const float* __restrict__ ref, const float* __restrict__ ref2,
    const float* __restrict__ scales, uint32_t* __restrict__ codes, uint64_t first_word, uint64_t d,
    uint64_t words, uint32_t M, float eps, uint32_t k0, uint32_t k1, uint32_t iter,
    const float* __restrict__ means, FusedScale fs) {
  constexpr int PER = 32 / BITS;
  const uint32_t m = blockIdx.y;
  const float mu = NORM == kNormMean ? means[m] : 0.f;
  const float R = fs.rows != 0 ? fused_scale(fs, m, M, blockIdx.x == 0 && threadIdx.x == 0) : scales[m];
  const float inv_r = R != 0.f ? 1.0f / R : 0.f;
  const uint64_t stride = (uint64_t)gridDim.x * kBlock;
  for (uint64_t wi = first_word + (uint64_t)blockIdx.x * kBlock + threadIdx.x; wi < words; wi += stride) {
    uint32_t word = 0u;
    if (R != 0.f) {
#pragma unroll 1
      for (int q = 0; q < PER / 4; ++q) {
        const uint64_t e0 = wi * PER + (uint64_t)q * 4;
        if (e0 >= d) break;
        const U32x4 rnd = philox4x32_10((uint32_t)(e0 >> 2), m, iter, 0u, k0, k1);
        const uint32_t rw[4] = {rnd.x, rnd.y, rnd.z, rnd.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const uint64_t e = e0 + k;
          if (e < d) {
            float r1, r2;
            load_ref_scalar<NORM>(ref, ref2, e, eps, r1, r2);
            const float v = normalize_w<NORM>(g[(uint64_t)m * d + e], r1, r2, mu);
            word |= quantize_code<BITS>(v, inv_r, rw[k]) << ((q * 4 + k) * BITS);
          }
        }
      }
    }
    codes[(uint64_t)m * words + wi] = word;
  }
}

// ------------------------------------------------------------------------------------------
// Server: decode, average over workers in worker order, de-normalise (Eq. 1 / Eq. 2), and
// optionally w <- w - lr * v and reference <- v in the same pass.
// ------------------------------------------------------------------------------------------
constexpr int kScaleChunk = 256;

template <int BITS>
__device__ __forceinline__ void stage_scales(const float* __restrict__ scales, uint32_t m_base, uint32_t M,
                                             float* sR, float* sStep) {
  constexpr float S = (float)((1 << (BITS - 1)) - 1);
  __syncthreads();
  if (threadIdx.x < kScaleChunk && m_base + threadIdx.x < M) {
    const float R = scales[m_base + threadIdx.x];
    sR[threadIdx.x] = R;
    sStep[threadIdx.x] = R / S;
  }
  __syncthreads();
}

// A workgroup owns a tile of kDecodeLoads * 256 float4 (4096 coordinates).  Per worker the tile's
// packed codes are 256 (ternary) or 512 (4-bit) consecutive words: each thread fetches one or two
// of them with coalesced streaming loads, kDecodeWorkers workers at a time, and the words are
// re-read from LDS as the 8- or 16-bit fragment belonging to each of the thread's float4 slots.
// A code is turned into its value by a per-worker table in LDS (2^BITS entries), which also maps
// the unused "sign with level 0" pattern to +0.
constexpr int kDecodeLoads = 4;
constexpr int kDecodeWorkers = 8;

template <int NORM, int BITS, int V, bool STREAM_CODES>
__global__ __launch_bounds__(kBlock) void decode_vec_kernel(
    const uint32_t* __restrict__ codes, const float* __restrict__ scales, const float4* ref4,
    const float4* __restrict__ ref24, float4* __restrict__ vbar4, float4* w4, float4* refout4,
    uint64_t nvec, uint64_t words, uint32_t M, float eps, float inv_m, float lr, const float* __restrict__ means) {
  constexpr int MCH = kDecodeWorkers;
  constexpr int FPW = 32 / (4 * BITS);     // 4-code fragments per packed word: 4 (ternary) or 2
  constexpr int WPT = (V + FPW - 1) / FPW; // packed words per thread and worker (some threads idle when V < FPW)
  constexpr int WORDS = kBlock * V / FPW;  // packed words per tile and worker
  constexpr int TAB = 1 << BITS;           // table entries per worker
  constexpr uint32_t MASK = (1u << BITS) - 1u;
  constexpr float S = (float)((1 << (BITS - 1)) - 1);
  __shared__ union {
    lds_u32 b32[MCH][WORDS];
    lds_u8 b8[MCH][WORDS * 4];
    lds_u16 b16[MCH][WORDS * 2];
  } buf;
  __shared__ float table[MCH * TAB];
  const uint64_t vec_base = (uint64_t)blockIdx.x * (kBlock * V);
  const uint64_t word_base = (uint64_t)blockIdx.x * WORDS;
  float4 acc[V];
#pragma unroll
  for (int v = 0; v < V; ++v) acc[v] = make_float4(0.f, 0.f, 0.f, 0.f);

  for (uint32_t m_base = 0; m_base < M; m_base += MCH) {
    const uint32_t cnt = min((uint32_t)MCH, M - m_base);
    uint32_t wreg[MCH][WPT];
#pragma unroll
    for (int mm = 0; mm < MCH; ++mm) {
#pragma unroll
      for (int k = 0; k < WPT; ++k) {
        const uint32_t wl = k * kBlock + threadIdx.x;   // word within the tile
        const uint64_t wi = word_base + wl;
        wreg[mm][k] = 0u;
        if ((uint32_t)mm < cnt && wl < (uint32_t)WORDS && wi < words)
          wreg[mm][k] = STREAM_CODES ? __builtin_nontemporal_load(codes + (uint64_t)(m_base + mm) * words + wi)
                                     : codes[(uint64_t)(m_base + mm) * words + wi];
      }
    }
    __syncthreads();  // the previous trip's LDS reads are done
#pragma unroll
    for (int mm = 0; mm < MCH; ++mm) {
#pragma unroll
      for (int k = 0; k < WPT; ++k)
        if (k * kBlock + threadIdx.x < (uint32_t)WORDS) buf.b32[mm][k * kBlock + threadIdx.x] = wreg[mm][k];
    }
    if (threadIdx.x < cnt * TAB) {
      const uint32_t mm = threadIdx.x / TAB, code = threadIdx.x % TAB;
      const float R = scales[m_base + mm];
      const float val = decode_code<BITS>(code, R, R / S);
      table[threadIdx.x] = NORM == kNormMean ? means[m_base + mm] + val : val;  // the worker's mean is added back
    }
    __syncthreads();
    for (uint32_t mm = 0; mm < cnt; ++mm) {
      const float* tab = table + mm * TAB;
#pragma unroll
      for (int v = 0; v < V; ++v) {
        const uint32_t f = BITS == 2 ? (uint32_t)buf.b8[mm][v * kBlock + threadIdx.x]
                                     : (uint32_t)buf.b16[mm][v * kBlock + threadIdx.x];
        acc[v].x = acc[v].x + tab[f & MASK];
        acc[v].y = acc[v].y + tab[(f >> BITS) & MASK];
        acc[v].z = acc[v].z + tab[(f >> (2 * BITS)) & MASK];
        acc[v].w = acc[v].w + tab[(f >> (3 * BITS)) & MASK];
      }
    }
  }

#pragma unroll
  for (int v = 0; v < V; ++v) {
    const uint64_t i = vec_base + (uint64_t)v * kBlock + threadIdx.x;
    if (i < nvec) {
      RefTile<NORM> rt;
      rt.load(ref4, ref24, i, eps);
      float4 o;
      o.x = denormalize<NORM>(acc[v].x * inv_m, rt.r1.x, rt.r2.x);
      o.y = denormalize<NORM>(acc[v].y * inv_m, rt.r1.y, rt.r2.y);
      o.z = denormalize<NORM>(acc[v].z * inv_m, rt.r1.z, rt.r2.z);
      o.w = denormalize<NORM>(acc[v].w * inv_m, rt.r1.w, rt.r2.w);
      store_stream(vbar4 + i, o);
      if (w4 != nullptr) {
        float4 w = load_stream(w4 + i);
        const float px = lr * o.x, py = lr * o.y, pz = lr * o.z, pw = lr * o.w;
        w.x = w.x - px;
        w.y = w.y - py;
        w.z = w.z - pz;
        w.w = w.w - pw;
        w4[i] = w;
      }
      if (refout4 != nullptr) refout4[i] = o;
    }
  }
}

// ------------------------------------------------------------------------------------------
// One workgroup for tiny problems (d <= 4 * kBlock): scale, quantise and pack, and (DECODE) the
// server side as well, in one launch.
//
// A thread owns one float4 of coordinates of every worker (M <= MC rows in registers), so once the
// M scales are known -- a workgroup reduction -- it can code its values, and since it then holds all
// M codes of its coordinates it can decode, average, de-normalise and update them without reading
// anything back.  Such problems are bound by the latency of their launches (about 4 us each), not
// by bytes.
// The same kernel over several workgroups, with the maxima exchanged through device-scope atomics
// and a meeting point (bounded wait, grid checked against the occupancy), was measured too: it wins
// up to 16 workgroups (16.6 -> 15.5 us per iteration at d = 2^14, M = 8) and loses beyond (d = 2^20,
// M = 8: 32 -> 56 us): with eight compute dies, each with its own L2, every arrival and every flag
// is an access to memory-side atomics, about 25 us for a full meeting of 128 or more workgroups.
// ------------------------------------------------------------------------------------------
constexpr int kSinglePassMaxWorkers = 16;

template <int NORM, int BITS, int MC, bool DECODE>
__global__ __launch_bounds__(kBlock) void single_pass_kernel(
    GradRows g, const float4* ref4, const float4* __restrict__ ref24, float* __restrict__ scales,
    uint32_t* __restrict__ codes, uint64_t nvec, uint64_t words, uint32_t M, float eps, uint32_t k0, uint32_t k1,
    uint32_t iter, float4* __restrict__ vbar4, float4* w4, float4* refout4, float inv_m, float lr) {
  constexpr int WPB = kBlock * 4 * BITS / 32;  // packed words per workgroup and worker
  constexpr uint32_t MASK = (1u << BITS) - 1u;
  constexpr float S = (float)((1 << (BITS - 1)) - 1);
  __shared__ float red[MC][kWavesPerBlock];
  __shared__ float sScale[MC];
  __shared__ union {
    lds_u8 b8[MC][WPB * 4];
    lds_u16 b16[MC][WPB * 2];
    lds_u32 b32[MC][WPB];
  } buf;
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const uint64_t q = threadIdx.x;  // one workgroup
  const bool active = q < nvec;

  RefTile<NORM> rt;
  rt.r1 = rt.r2 = make_float4(0.f, 0.f, 0.f, 0.f);
  float4 x[MC];
  float amax[MC];
  if (active) {
    rt.template load<false>(ref4, ref24, q, eps);
#pragma unroll
    for (int mm = 0; mm < MC; ++mm)  // rows past M repeat the last one: all loads in flight, none under a condition
      x[mm] = load_row_stream(g.row(min((uint32_t)mm, M - 1)) + q);
  }
#pragma unroll
  for (int mm = 0; mm < MC; ++mm) {
    amax[mm] = 0.f;
    if (active) {
      const float a0 = fabsf(normalize<NORM>(x[mm].x, rt.r1.x, rt.r2.x));
      const float a1 = fabsf(normalize<NORM>(x[mm].y, rt.r1.y, rt.r2.y));
      const float a2 = fabsf(normalize<NORM>(x[mm].z, rt.r1.z, rt.r2.z));
      const float a3 = fabsf(normalize<NORM>(x[mm].w, rt.r1.w, rt.r2.w));
      amax[mm] = fmaxf(fmaxf(a0, a1), fmaxf(a2, a3));
    }
    const float v = wave_max(amax[mm]);
    if (lane == 0) red[mm][wave] = v;
  }
  __syncthreads();
  if (threadIdx.x < M) {
    float v = red[threadIdx.x][0];
#pragma unroll
    for (int k = 1; k < kWavesPerBlock; ++k) v = fmaxf(v, red[threadIdx.x][k]);
    v = v < FLT_MIN ? 0.f : v;
    sScale[threadIdx.x] = v;
    scales[threadIdx.x] = v;
  }
  __syncthreads();

  uint32_t frag[MC];
#pragma unroll
  for (int mm = 0; mm < MC; ++mm) {
    frag[mm] = 0u;
    if ((uint32_t)mm < M) {
      const float R = sScale[mm];
      if (active && R != 0.f) {
        const float inv_r = 1.0f / R;
        const U32x4 rnd = philox4x32_10((uint32_t)q, (uint32_t)mm, iter, 0u, k0, k1);
        const uint32_t c0 = quantize_code<BITS>(normalize<NORM>(x[mm].x, rt.r1.x, rt.r2.x), inv_r, rnd.x);
        const uint32_t c1 = quantize_code<BITS>(normalize<NORM>(x[mm].y, rt.r1.y, rt.r2.y), inv_r, rnd.y);
        const uint32_t c2 = quantize_code<BITS>(normalize<NORM>(x[mm].z, rt.r1.z, rt.r2.z), inv_r, rnd.z);
        const uint32_t c3 = quantize_code<BITS>(normalize<NORM>(x[mm].w, rt.r1.w, rt.r2.w), inv_r, rnd.w);
        frag[mm] = c0 | (c1 << BITS) | (c2 << (2 * BITS)) | (c3 << (3 * BITS));
      }
      if (BITS == 2) {
        buf.b8[mm][threadIdx.x] = (uint8_t)frag[mm];
      } else {
        buf.b16[mm][threadIdx.x] = (uint16_t)frag[mm];
      }
    }
  }
  __syncthreads();
  for (uint32_t t = threadIdx.x; t < M * (uint32_t)WPB; t += kBlock) {
    const uint32_t mm = t / WPB, j = t % WPB;
    const uint64_t wi = j;
    if (wi < words) store_word_through(codes + (uint64_t)mm * words + wi, buf.b32[mm][j]);
  }

  if (DECODE && active) {
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int mm = 0; mm < MC; ++mm) {
      if ((uint32_t)mm < M) {
        const float R = sScale[mm], step = R / S;
        const uint32_t f = frag[mm];
        acc.x = acc.x + decode_code<BITS>(f & MASK, R, step);
        acc.y = acc.y + decode_code<BITS>((f >> BITS) & MASK, R, step);
        acc.z = acc.z + decode_code<BITS>((f >> (2 * BITS)) & MASK, R, step);
        acc.w = acc.w + decode_code<BITS>((f >> (3 * BITS)) & MASK, R, step);
      }
    }
    float4 o;
    o.x = denormalize<NORM>(acc.x * inv_m, rt.r1.x, rt.r2.x);
    o.y = denormalize<NORM>(acc.y * inv_m, rt.r1.y, rt.r2.y);
    o.z = denormalize<NORM>(acc.z * inv_m, rt.r1.z, rt.r2.z);
    o.w = denormalize<NORM>(acc.w * inv_m, rt.r1.w, rt.r2.w);
    store_stream(vbar4 + q, o);
    if (w4 != nullptr) {
      float4 w = load_stream(w4 + q);
      const float px = lr * o.x, py = lr * o.y, pz = lr * o.z, pw = lr * o.w;
      w.x = w.x - px;
      w.y = w.y - py;
      w.z = w.z - pz;
      w.w = w.w - pw;
      w4[q] = w;
    }
    if (refout4 != nullptr) refout4[q] = o;
  }
}

template <int NORM, int BITS>
__global__ __launch_bounds__(kBlock) void decode_scalar_kernel(
    const uint32_t* __restrict__ codes, const float* __restrict__ scales, const float* ref,
    const float* __restrict__ ref2, float* __restrict__ vbar, float* __restrict__ w, float* refout, uint64_t first,
    uint64_t d, uint64_t words, uint32_t M, float eps, float inv_m, float lr, const float* __restrict__ means) {
  __shared__ float sR[kScaleChunk], sStep[kScaleChunk];
  constexpr int PER = 32 / BITS;
  constexpr uint32_t MASK = (1u << BITS) - 1u;
  const uint64_t e = first + (uint64_t)blockIdx.x * kBlock + threadIdx.x;
  const bool active = e < d;
  const uint64_t wi = e / PER;
  const uint32_t sh = (uint32_t)(e % PER) * BITS;
  float acc = 0.f;
  for (uint32_t m_base = 0; m_base < M; m_base += kScaleChunk) {
    stage_scales<BITS>(scales, m_base, M, sR, sStep);
    if (active) {
      const uint32_t cnt = min((uint32_t)kScaleChunk, M - m_base);
      for (uint32_t mm = 0; mm < cnt; ++mm) {
        const uint32_t word = codes[(uint64_t)(m_base + mm) * words + wi];
        const float val = decode_code<BITS>((word >> sh) & MASK, sR[mm], sStep[mm]);
        acc = acc + (NORM == kNormMean ? means[m_base + mm] + val : val);
      }
    }
  }
  if (!active) return;
  float r1, r2;
  load_ref_scalar<NORM>(ref, ref2, e, eps, r1, r2);
  const float v = denormalize<NORM>(acc * inv_m, r1, r2);
  vbar[e] = v;
  if (w != nullptr) {
    const float p = lr * v;
    w[e] = w[e] - p;
  }
  if (refout != nullptr) refout[e] = v;
}

// ------------------------------------------------------------------------------------------
// Order-pinned float64 sums per worker: the mean of the per-worker mean reference (section
// "Reference Vectors", first option) and the l2 norm as the coder's scale.
// ------------------------------------------------------------------------------------------
// The sum of a row is defined with a fixed association so that its float32 rounding is reproducible:
// elements are cut into chunks of 4096; inside a chunk lane j (0..255) adds the elements 256 k + j,
// k = 0..15 in order, and the 256 lane sums are added in lane order; chunk sums are added in order
// inside groups of 256 chunks, group sums in order.  One wavefront owns a chunk: thread t holds
// lanes 4t..4t+3 (one float4 per k), so every load instruction covers 1 KiB of contiguous memory.
constexpr int kTreeChunk = 4096;
constexpr int kTreeLanes = 256;
constexpr int kTreeGroup = 256;

// MINMAX (mean pass only): the smallest and largest element of every chunk ride along.  Rounding is
// monotone, so max_e |fl(g_e - mu)| = max(|fl(min g - mu)|, |fl(max g - mu)|) exactly: the scale of
// the mean-referenced gradient needs no pass of its own.
template <int NORM, bool SQUARE, bool VEC, bool MINMAX>
__global__ __launch_bounds__(kBlock) void tree_chunk_kernel(const float* __restrict__ g, const float* __restrict__ ref,
                                                            const float* __restrict__ ref2,
                                                            const float* __restrict__ means,
                                                            double* __restrict__ chunk_sums,
                                                            float2* __restrict__ chunk_minmax, uint64_t d,
                                                            uint64_t first_chunk, uint64_t end_chunk,
                                                            uint64_t nchunks, float eps, uint32_t M,
                                                            uint32_t workers_per_block) {
  __shared__ double lanes[kWavesPerBlock][kTreeLanes];
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const uint64_t chunk = first_chunk + (uint64_t)blockIdx.x * kWavesPerBlock + wave;
  if (chunk >= end_chunk) return;  // whole wavefront; no workgroup barrier below
  const uint64_t base = chunk * kTreeChunk + 4u * (uint32_t)lane;
  constexpr int K = kTreeChunk / kTreeLanes;
  // A wavefront takes its chunk of several workers in turn: the reference tile of the chunk is then
  // fetched from HBM once and found in cache by the following workers.
  const uint32_t m_first = blockIdx.y * workers_per_block;
  const uint32_t m_last = m_first + workers_per_block < M ? m_first + workers_per_block : M;
  for (uint32_t m = m_first; m < m_last; ++m) {
  const float* __restrict__ row = g + (uint64_t)m * d;
  const float mu = (SQUARE && NORM == kNormMean) ? means[m] : 0.f;
  double acc[4] = {0.0, 0.0, 0.0, 0.0};
  float lo = INFINITY, hi = -INFINITY;
  // VEC: 16-byte loads (the row may start at any 4-byte boundary).  The caller keeps the last chunk of
  // rows whose length is not a multiple of 4 away from this variant.
  if (VEC) {
    const bool full = (chunk + 1) * kTreeChunk <= d;
    // loads in batches: all 16 rows of the chunk at once, or 8 rows plus their reference tiles
    constexpr bool kHasRef = SQUARE && (NORM == kNormSub || NORM == kNormQuot || NORM == kNormComb);
    constexpr int KB = kHasRef ? 8 : K;
#pragma unroll
    for (int k0 = 0; k0 < K; k0 += KB) {
      float4 x[KB];
      RefTile<NORM> rt[KB];
#pragma unroll
      for (int k = 0; k < KB; ++k) {
        const uint64_t e = base + (uint64_t)(k0 + k) * kTreeLanes;
        const bool in = full || e < d;
        x[k] = in ? load_row_stream(reinterpret_cast<const v4f_u_t*>(row + e)) : make_float4(0.f, 0.f, 0.f, 0.f);
        if (SQUARE && in)
          rt[k].template load<false>(reinterpret_cast<const float4*>(ref), reinterpret_cast<const float4*>(ref2), e / 4,
                                     eps);
      }
#pragma unroll
      for (int k = 0; k < KB; ++k) {
        const uint64_t e = base + (uint64_t)(k0 + k) * kTreeLanes;
        const bool in = full || e < d;
        float4 v = x[k];
        if (SQUARE && in) {
          v.x = normalize_w<NORM>(v.x, rt[k].r1.x, rt[k].r2.x, mu);
          v.y = normalize_w<NORM>(v.y, rt[k].r1.y, rt[k].r2.y, mu);
          v.z = normalize_w<NORM>(v.z, rt[k].r1.z, rt[k].r2.z, mu);
          v.w = normalize_w<NORM>(v.w, rt[k].r1.w, rt[k].r2.w, mu);
        }
        if (MINMAX && in) {
          lo = fminf(lo, fminf(fminf(v.x, v.y), fminf(v.z, v.w)));
          hi = fmaxf(hi, fmaxf(fmaxf(v.x, v.y), fmaxf(v.z, v.w)));
        }
        const double t0 = (double)v.x, t1 = (double)v.y, t2 = (double)v.z, t3 = (double)v.w;
        acc[0] = acc[0] + (SQUARE ? t0 * t0 : t0);  // the square of a binary32 value is exact in binary64
        acc[1] = acc[1] + (SQUARE ? t1 * t1 : t1);
        acc[2] = acc[2] + (SQUARE ? t2 * t2 : t2);
        acc[3] = acc[3] + (SQUARE ? t3 * t3 : t3);
      }
    }
  } else {
    for (int k = 0; k < K; ++k) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint64_t e = base + (uint64_t)k * kTreeLanes + i;
        if (e < d) {
          float v = row[e];
          if (SQUARE) {
            float r1, r2;
            load_ref_scalar<NORM>(ref, ref2, e, eps, r1, r2);
            v = normalize_w<NORM>(v, r1, r2, mu);
          }
          if (MINMAX) {
            lo = fminf(lo, v);
            hi = fmaxf(hi, v);
          }
          const double t = (double)v;
          acc[i] = acc[i] + (SQUARE ? t * t : t);
        }
      }
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) lanes[wave][4 * lane + i] = acc[i];
  if (MINMAX) {
    hi = wave_max(hi);
    lo = -wave_max(-lo);
  }
  wave_lds_fence();
  if (lane == 0) {
    double total = 0.0;
#pragma unroll 16
    for (int j = 0; j < kTreeLanes; ++j) total = total + lanes[wave][j];
    chunk_sums[(uint64_t)m * nchunks + chunk] = total;
    if (MINMAX) chunk_minmax[(uint64_t)m * nchunks + chunk] = make_float2(lo, hi);
  }
  wave_lds_fence();  // the lane sums are read before the next worker overwrites them
  }
}

// Chunk sums of the squares for the normalisations with a shared reference, whole chunks only: the
// reference tile of a quarter chunk stays in registers while MC workers use it (as in the maximum
// pass), so the reference is read from memory once per MC workers.  Lane sums still add their
// elements in the order k = 0..15: the quarters and the rows inside a quarter are walked in order.
template <int NORM, int MC>
__global__ __launch_bounds__(kBlock) void l2_chunk_kernel(GradRows g, const float4* __restrict__ ref4,
                                                          const float4* __restrict__ ref24,
                                                          double* __restrict__ chunk_sums, uint64_t whole_chunks,
                                                          uint64_t nchunks, float eps, uint32_t M) {
  __shared__ double lanes[kWavesPerBlock][kTreeLanes];
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const uint64_t chunk = (uint64_t)blockIdx.x * kWavesPerBlock + wave;
  if (chunk >= whole_chunks) return;  // whole wavefront; no workgroup barrier below
  const uint32_t m0 = blockIdx.y * MC;
  constexpr int Q = 4;                                  // rows (k) per quarter chunk
  constexpr int K = kTreeChunk / kTreeLanes;            // 16 rows of 64 float4 per chunk
  const uint64_t v0 = chunk * (kTreeChunk / 4) + lane;  // float4 index of row k = 0
  double acc[MC][4];
#pragma unroll
  for (int mm = 0; mm < MC; ++mm) acc[mm][0] = acc[mm][1] = acc[mm][2] = acc[mm][3] = 0.0;
#pragma unroll 1
  for (int k0 = 0; k0 < K; k0 += Q) {
    RefTile<NORM> rt[Q];
#pragma unroll
    for (int k = 0; k < Q; ++k) rt[k].load(ref4, ref24, v0 + (uint64_t)(k0 + k) * kWave, eps);
#pragma unroll
    for (int mm = 0; mm < MC; ++mm) {
      // rows past M (MC not dividing M) repeat the last row; their sums are not stored
      const v4f_u_t* __restrict__ row = g.row(min(m0 + (uint32_t)mm, M - 1));
      float4 x[Q];
#pragma unroll
      for (int k = 0; k < Q; ++k) x[k] = load_row_stream(row + v0 + (uint64_t)(k0 + k) * kWave);
#pragma unroll
      for (int k = 0; k < Q; ++k) {
        const double t0 = (double)normalize<NORM>(x[k].x, rt[k].r1.x, rt[k].r2.x);
        const double t1 = (double)normalize<NORM>(x[k].y, rt[k].r1.y, rt[k].r2.y);
        const double t2 = (double)normalize<NORM>(x[k].z, rt[k].r1.z, rt[k].r2.z);
        const double t3 = (double)normalize<NORM>(x[k].w, rt[k].r1.w, rt[k].r2.w);
        acc[mm][0] = acc[mm][0] + t0 * t0;  // the square of a binary32 value is exact in binary64
        acc[mm][1] = acc[mm][1] + t1 * t1;
        acc[mm][2] = acc[mm][2] + t2 * t2;
        acc[mm][3] = acc[mm][3] + t3 * t3;
      }
    }
  }
#pragma unroll
  for (int mm = 0; mm < MC; ++mm) {
#pragma unroll
    for (int i = 0; i < 4; ++i) lanes[wave][4 * lane + i] = acc[mm][i];
    wave_lds_fence();
    if (lane == 0 && m0 + mm < M) {
      double total = 0.0;
#pragma unroll 16
      for (int j = 0; j < kTreeLanes; ++j) total = total + lanes[wave][j];
      chunk_sums[(uint64_t)(m0 + mm) * nchunks + chunk] = total;
    }
    wave_lds_fence();
  }
}

// One workgroup per worker: group sums (thread q adds the chunks of groups q, q + 256, ... in order),
// then thread 0 adds the groups in order.  MEAN: out[m] = float(total / d), and, when chunk_minmax is
// given, scales[m] = max |g - out[m]| from the smallest and the largest element.  Otherwise
// out[m] = float(sqrt(total)), 0 when below FLT_MIN.  Division and square root of binary64 are
// correctly rounded on the device, so the float32 result is the same as on any IEEE host.
template <bool MEAN>
__global__ __launch_bounds__(kBlock) void tree_finish_kernel(const double* __restrict__ chunk_sums,
                                                             double* __restrict__ group_sums,
                                                             const float2* __restrict__ chunk_minmax,
                                                             uint64_t nchunks, uint64_t ngroups, uint64_t d,
                                                             float* __restrict__ out, float* __restrict__ scales) {
  __shared__ float red_lo[kWavesPerBlock], red_hi[kWavesPerBlock];
  const uint32_t m = blockIdx.x;
  const double* __restrict__ cs = chunk_sums + (uint64_t)m * nchunks;
  double* __restrict__ gs = group_sums + (uint64_t)m * ngroups;
  for (uint64_t q = threadIdx.x; q < ngroups; q += kBlock) {
    const uint64_t c0 = q * kTreeGroup;
    const uint64_t c1 = c0 + kTreeGroup < nchunks ? c0 + kTreeGroup : nchunks;
    double a = 0.0;
    for (uint64_t c = c0; c < c1; ++c) a = a + cs[c];
    gs[q] = a;
  }
  if (MEAN && chunk_minmax != nullptr) {
    float lo = INFINITY, hi = -INFINITY;
    for (uint64_t c = threadIdx.x; c < nchunks; c += kBlock) {
      const float2 mm = chunk_minmax[(uint64_t)m * nchunks + c];
      lo = fminf(lo, mm.x);
      hi = fmaxf(hi, mm.y);
    }
    lo = -wave_max(-lo);
    hi = wave_max(hi);
    if (threadIdx.x % kWave == 0) {
      red_lo[threadIdx.x / kWave] = lo;
      red_hi[threadIdx.x / kWave] = hi;
    }
  }
  __threadfence_block();
  __syncthreads();
  if (threadIdx.x == 0) {
    double total = 0.0;
    for (uint64_t q = 0; q < ngroups; ++q) total = total + gs[q];
    if (MEAN) {
      const float mu = (float)(total / (double)d);
      out[m] = mu;
      if (chunk_minmax != nullptr) {
        float lo = red_lo[0], hi = red_hi[0];
#pragma unroll
        for (int k = 1; k < kWavesPerBlock; ++k) {
          lo = fminf(lo, red_lo[k]);
          hi = fmaxf(hi, red_hi[k]);
        }
        const float r = fmaxf(fabsf(lo - mu), fabsf(hi - mu));
        scales[m] = r < FLT_MIN ? 0.f : r;
      }
    } else {
      const float r = (float)sqrt(total);
      out[m] = r < FLT_MIN ? 0.f : r;
    }
  }
}

// ------------------------------------------------------------------------------------------
// Launch geometry
// ------------------------------------------------------------------------------------------
inline uint32_t div_up_u32(uint64_t a, uint64_t b) {
  const uint64_t q = (a + b - 1) / b;
  return (uint32_t)(q > kMaxGridX ? kMaxGridX : q);
}

// Workers handled inside one workgroup (8, 4, 2 or 1; the last group of a row of workgroups may be
// short).  A group reads the shared reference once, so fewer groups mean less traffic; a short group
// costs the scale pass repeated loads of its last row (cache hits: repeat_cost 0.3 of a row there,
// nothing in the quantiser, which stops at the last worker).  At least 2048 workgroups are kept to
// fill 256 compute units.
inline int pick_workers_per_block(uint32_t M, uint64_t tiles, double repeat_cost, int mc_max = 8) {
  int best = 1;
  double best_cost = (double)M;
  for (int mc = 2; mc <= mc_max; mc *= 2) {
    const uint32_t groups = (M + mc - 1) / mc;
    if (tiles * groups < 2048 || (mc > 8 && M <= 8)) break;
    const double cost = groups + repeat_cost * (groups * mc - M);
    if (cost <= best_cost) {
      best = mc;
      best_cost = cost;
    }
  }
  return best;
}

// How many leading coordinates of every row the vector kernels take: all of them when d is a
// multiple of 4, else the largest multiple of 16 (whole packed words for either code width); the
// scalar kernels finish the rest of each row.  0: scalar kernels only (the shared operands are not
// 16-byte aligned).
inline bool aligned16_or_null(const void* a, const void* b, const void* c = nullptr, const void* e = nullptr) {
  auto al = [](const void* p) { return p == nullptr || (reinterpret_cast<uintptr_t>(p) & 15u) == 0; };
  return al(a) && al(b) && al(c) && al(e);
}
inline uint64_t vector_part(uint64_t d, const void* a, const void* b, const void* c = nullptr,
                            const void* e = nullptr) {
  if (!aligned16_or_null(a, b, c, e)) return 0;
  return d % 4 == 0 ? d : d - d % 16;
}

inline bool vec_ok(uint64_t d, const void* a, const void* b, const void* c) {
  auto al = [](const void* p) { return p == nullptr || (reinterpret_cast<uintptr_t>(p) & 15u) == 0; };
  return d % 4 == 0 && al(a) && al(b) && al(c);
}

template <int NORM, int MC>
hipError_t absmax_vec_launch(const CodecShape& c, uint64_t dv, const float* g, const float* gref, const float* gref2,
                             float* partials, uint32_t* nblocks, hipStream_t s) {
  const uint64_t nvec = dv / 4;
  const uint32_t per_y = div_up_u32(nvec, (uint64_t)kBlock * kAbsmaxLoads);
  const uint32_t cap = kAbsmaxMaxBlocks - 1;  // one row of partials is kept for the rows' scalar remainder
  const uint32_t gx = per_y < cap ? per_y : cap;
  *nblocks = gx;
  dim3 grid(gx, (c.M + MC - 1) / MC);
  hipLaunchKernelGGL((absmax_vec_kernel<NORM, MC>), grid, dim3(kBlock), 0, s, GradRows{g, c.d},
                     reinterpret_cast<const float4*>(gref), reinterpret_cast<const float4*>(gref2), partials, nvec,
                     c.M, c.eps, c.means);
  return hipGetLastError();
}

// Scratch of the ternary coder that reads g once: the word that says whether the slots are used, the
// sample's maxima [M], the sample pass's partial maxima [kAbsmaxMaxBlocks][M], the overflow counts of the
// scale pass's workgroups (as many), the slots [M][d / 1024] of 1 KiB.
struct CandidateScratch {
  uint32_t* use_slots;
  float* sample_max;
  uint32_t* select_ok;
  float* sample_partials;
  float* sample_sums;
  uint32_t* overflowed;
  uint32_t* slots;
};
inline size_t round_up_256(size_t v) { return (v + 255) / 256 * 256; }
inline size_t candidate_head_bytes(uint32_t M) {
  return 256 + 2 * round_up_256((size_t)M * sizeof(float)) + 3 * round_up_256((size_t)kAbsmaxMaxBlocks * M * sizeof(float));
}
inline CandidateScratch candidate_scratch(const CodecShape& c, void* scratch) {
  unsigned char* p = static_cast<unsigned char*>(scratch);
  CandidateScratch cs;
  cs.use_slots = reinterpret_cast<uint32_t*>(p);
  p += 256;
  cs.sample_max = reinterpret_cast<float*>(p);
  p += round_up_256((size_t)c.M * sizeof(float));
  cs.select_ok = reinterpret_cast<uint32_t*>(p);
  p += round_up_256((size_t)c.M * sizeof(float));
  cs.sample_partials = reinterpret_cast<float*>(p);
  p += round_up_256((size_t)kAbsmaxMaxBlocks * c.M * sizeof(float));
  cs.sample_sums = reinterpret_cast<float*>(p);
  p += round_up_256((size_t)kAbsmaxMaxBlocks * c.M * sizeof(float));
  cs.overflowed = reinterpret_cast<uint32_t*>(p);
  p += round_up_256((size_t)kAbsmaxMaxBlocks * c.M * sizeof(float));
  cs.slots = reinterpret_cast<uint32_t*>(p);
  return cs;
}

template <int NORM>
hipError_t absmax_candidates_dispatch(const CodecShape& c, uint32_t iter, const float* g, const float* gref,
                                      const float* gref2, float* partials, const CandidateScratch& cs, float* scales,
                                      hipStream_t s) {
  const uint64_t nvec = c.d / 4;
  const int mc = pick_workers_per_block(c.M, (nvec + kBlock * kAbsmaxLoads - 1) / (kBlock * kAbsmaxLoads), 0.3);
  uint32_t nblocks = 0;
  hipError_t e;
  // the sample: every kSampleStride-th wavefront tile of every row
  const uint64_t row_tiles = nvec / (kWave * kAbsmaxLoads);
  const uint64_t sample_tiles = (row_tiles + kSampleStride - 1) / kSampleStride;
  uint32_t nsample = div_up_u32(sample_tiles, kWavesPerBlock);
  if (nsample > kAbsmaxMaxBlocks) nsample = kAbsmaxMaxBlocks;
  hipLaunchKernelGGL((sample_stats_kernel<NORM>), dim3(nsample, c.M), dim3(kBlock), 0, s, GradRows{g, c.d},
                     reinterpret_cast<const float4*>(gref), cs.sample_partials, cs.sample_sums, nvec, c.M);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(sample_finish_kernel, dim3(c.M), dim3(kBlock), 0, s, cs.sample_partials, cs.sample_sums, nsample,
                     c.M, (float)(sample_tiles * (kWave * kAbsmaxLoads * 4)), cs.sample_max, cs.select_ok);
  const uint32_t per_y = div_up_u32(nvec, (uint64_t)kBlock * kAbsmaxLoads);
  const uint32_t cap = kAbsmaxMaxBlocks - 1;
  nblocks = per_y < cap ? per_y : cap;
#define TNG_SELECT(MC)                                                                                              \
  hipLaunchKernelGGL((absmax_select_kernel<NORM, MC>), dim3(nblocks, (c.M + MC - 1) / MC), dim3(kBlock), 0, s,      \
                     GradRows{g, c.d}, reinterpret_cast<const float4*>(gref), reinterpret_cast<const float4*>(gref2), \
                     partials, nvec, c.M, c.eps, cs.sample_max, cs.select_ok, cs.slots, cs.overflowed, c.k0, c.k1, iter)
  switch (mc) {
    case 8: TNG_SELECT(8); break;
    case 4: TNG_SELECT(4); break;
    case 2: TNG_SELECT(2); break;
    default: TNG_SELECT(1); break;
  }
#undef TNG_SELECT
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(absmax_finish_vote_kernel, dim3(c.M + 1), dim3(kBlock), 0, s, partials, nblocks, c.M, scales,
                     cs.overflowed, nblocks * ((c.M + (uint32_t)mc - 1) / (uint32_t)mc),
                     (uint64_t)c.M * (nvec / (kWave * kAbsmaxLoads)), cs.use_slots);
  return hipGetLastError();
}

template <int NORM, int BITS>
hipError_t quantize_dispatch(const CodecShape& c, uint32_t iter, const float* g, const float* gref,
                             const float* gref2, float* scales, uint32_t* codes, const float* partials,
                             uint32_t fused_rows, hipStream_t s, const uint32_t* skip_if_set = nullptr);

template <int NORM>
hipError_t quantize_candidates_dispatch(const CodecShape& c, uint32_t iter, const float* g, const float* gref,
                                        const float* gref2, const float* scales, const CandidateScratch& cs,
                                        uint32_t* codes, hipStream_t s) {
  const uint64_t nvec = c.d / 4;
  const uint64_t tiles = (nvec + kBlock * kLoadsPerLane - 1) / (kBlock * kLoadsPerLane);  // workgroups of 4 wavefront tiles
  const int mc = pick_workers_per_block(c.M, tiles, 0.0, 16);
#define TNG_QC(MC)                                                                                                   \
  hipLaunchKernelGGL((quantize_candidates_kernel<NORM, MC>), dim3((uint32_t)tiles, (c.M + MC - 1) / MC), dim3(kBlock), 0, \
                     s, GradRows{g, c.d}, reinterpret_cast<const float4*>(gref), reinterpret_cast<const float4*>(gref2), \
                     scales, cs.slots, codes, nvec, c.words, c.M, c.eps, c.k0, c.k1, iter, cs.use_slots, cs.select_ok)
  switch (mc) {
    case 16: TNG_QC(16); break;
    case 8: TNG_QC(8); break;
    case 4: TNG_QC(4); break;
    case 2: TNG_QC(2); break;
    default: TNG_QC(1); break;
  }
#undef TNG_QC
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  // the ordinary quantiser right behind it: one of the two returns at once, by the vote of the scale pass
  return quantize_dispatch<NORM, 2>(c, iter, g, gref, gref2, const_cast<float*>(scales), codes, nullptr, 0, s,
                                    cs.use_slots);
}

template <int NORM>
hipError_t absmax_dispatch(const CodecShape& c, const float* g, const float* gref, const float* gref2,
                           float* partials, float* scales, hipStream_t s) {
  uint32_t nblocks = 0;
  hipError_t e;
  const uint64_t dv = vector_part(c.d, gref, gref2);
  if (dv != 0) {
    const int mc = pick_workers_per_block(c.M, (dv / 4 + kBlock * kAbsmaxLoads - 1) / (kBlock * kAbsmaxLoads), 0.3);
    switch (mc) {
      case 8: e = absmax_vec_launch<NORM, 8>(c, dv, g, gref, gref2, partials, &nblocks, s); break;
      case 4: e = absmax_vec_launch<NORM, 4>(c, dv, g, gref, gref2, partials, &nblocks, s); break;
      case 2: e = absmax_vec_launch<NORM, 2>(c, dv, g, gref, gref2, partials, &nblocks, s); break;
      default: e = absmax_vec_launch<NORM, 1>(c, dv, g, gref, gref2, partials, &nblocks, s); break;
    }
    if (e == hipSuccess && dv < c.d) {  // the last d - dv < 16 coordinates of every row: one more row of partials
      hipLaunchKernelGGL((absmax_scalar_kernel<NORM>), dim3(1, c.M), dim3(kBlock), 0, s, g, gref, gref2,
                         partials + (uint64_t)nblocks * c.M, dv, c.d, c.M, c.eps, c.means);
      nblocks += 1;
      e = hipGetLastError();
    }
  } else {
    const uint32_t per_y = div_up_u32(c.d, kBlock);
    nblocks = per_y < kAbsmaxMaxBlocks ? per_y : kAbsmaxMaxBlocks;
    hipLaunchKernelGGL((absmax_scalar_kernel<NORM>), dim3(nblocks, c.M), dim3(kBlock), 0, s, g, gref, gref2,
                       partials, (uint64_t)0, c.d, c.M, c.eps, c.means);
    e = hipGetLastError();
  }
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(absmax_finish_kernel, dim3(c.M), dim3(kBlock), 0, s, partials, nblocks, c.M, scales);
  return hipGetLastError();
}

template <int NORM, int BITS, int MC, bool FUSED>
hipError_t quantize_vec_launch(const CodecShape& c, uint64_t dv, uint32_t iter, const float* g, const float* gref,
                               const float* gref2, const float* scales, uint32_t* codes, const FusedScale& fs,
                               hipStream_t s, const uint32_t* skip_if_set = nullptr) {
  const uint64_t nvec = dv / 4;
  const uint64_t tiles = (nvec + kBlock * kLoadsPerLane - 1) / (kBlock * kLoadsPerLane);
  dim3 grid((uint32_t)tiles, (c.M + MC - 1) / MC);
  hipLaunchKernelGGL((quantize_pack_vec_kernel<NORM, BITS, MC, FUSED>), grid, dim3(kBlock), 0, s, GradRows{g, c.d},
                     reinterpret_cast<const float4*>(gref), reinterpret_cast<const float4*>(gref2), scales, codes, nvec,
                     c.words, c.M, c.eps, c.k0, c.k1, iter, c.means, fs, skip_if_set);
  return hipGetLastError();
}

// fused_rows > 0: scales is an output and the scale is taken from the first fused_rows rows of
// partials (see FusedScale); only problems small enough for one worker per workgroup go that way,
// larger ones get the reduction kernel first.
template <int NORM, int BITS>
hipError_t quantize_dispatch(const CodecShape& c, uint32_t iter, const float* g, const float* gref,
                             const float* gref2, float* scales, uint32_t* codes, const float* partials,
                             uint32_t fused_rows, hipStream_t s, const uint32_t* skip_if_set) {
  const uint64_t dv = vector_part(c.d, gref, gref2);
  const bool vec = dv != 0;
  const uint64_t tiles = (dv / 4 + kBlock * kLoadsPerLane - 1) / (kBlock * kLoadsPerLane);
  const int mc = vec ? pick_workers_per_block(c.M, tiles, 0.0, 16) : 1;
  FusedScale fs{partials, fused_rows, scales};
  if (fused_rows > kFusedScaleRows || (fused_rows > 0 && (mc != 1 || dv != c.d))) {
    hipLaunchKernelGGL(absmax_finish_kernel, dim3(c.M), dim3(kBlock), 0, s, partials, fused_rows, c.M, scales);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    fs.rows = 0;
  }
  if (vec) {
    hipError_t e;
    if (fs.rows > 0) {
      e = quantize_vec_launch<NORM, BITS, 1, true>(c, dv, iter, g, gref, gref2, scales, codes, fs, s);
    } else {
      switch (mc) {
        case 16: e = quantize_vec_launch<NORM, BITS, 16, false>(c, dv, iter, g, gref, gref2, scales, codes, fs, s, skip_if_set); break;
        case 8: e = quantize_vec_launch<NORM, BITS, 8, false>(c, dv, iter, g, gref, gref2, scales, codes, fs, s, skip_if_set); break;
        case 4: e = quantize_vec_launch<NORM, BITS, 4, false>(c, dv, iter, g, gref, gref2, scales, codes, fs, s, skip_if_set); break;
        case 2: e = quantize_vec_launch<NORM, BITS, 2, false>(c, dv, iter, g, gref, gref2, scales, codes, fs, s, skip_if_set); break;
        default: e = quantize_vec_launch<NORM, BITS, 1, false>(c, dv, iter, g, gref, gref2, scales, codes, fs, s, skip_if_set); break;
      }
    }
    if (e != hipSuccess || dv == c.d) return e;
    // the last d - dv < 16 coordinates of every row: their one or two packed words, after the vector pass
    hipLaunchKernelGGL((quantize_pack_scalar_kernel<NORM, BITS>), dim3(1, c.M), dim3(kBlock), 0, s, g, gref, gref2,
                       scales, codes, dv * BITS / 32, c.d, c.words, c.M, c.eps, c.k0, c.k1, iter, c.means, fs);
    return hipGetLastError();
  }
  const uint32_t per_y = div_up_u32(c.words, kBlock);
  dim3 grid(per_y < 65536u ? per_y : 65536u, c.M);
  hipLaunchKernelGGL((quantize_pack_scalar_kernel<NORM, BITS>), grid, dim3(kBlock), 0, s, g, gref, gref2,
                     scales, codes, (uint64_t)0, c.d, c.words, c.M, c.eps, c.k0, c.k1, iter, c.means, fs);
  return hipGetLastError();
}

template <int NORM, int BITS>
hipError_t decode_dispatch(const CodecShape& c, const uint32_t* codes, const float* scales, const float* gref,
                           const float* gref2, float* vbar, float* w, float lr, float* ref_out,
                           hipStream_t s) {
  const float inv_m = 1.0f / (float)c.M;
  const uint64_t dv = vector_part(c.d, gref, gref2, vbar, w) != 0 ? vector_part(c.d, ref_out, nullptr) : 0;
  if (dv != 0) {
    const uint64_t nvec = dv / 4;
    const uint64_t big_tiles = (nvec + kBlock * kDecodeLoads - 1) / (kBlock * kDecodeLoads);
    // Codes that fit the 256 MiB last-level cache were just written by the quantiser and are rewritten
    // by the next iteration: ordinary loads keep the lines resident (measured 4 % faster, and the
    // following quantise pass too); larger code arrays are streamed (measured 17 % faster at 512 MiB).
    const bool stream_codes = (uint64_t)c.M * c.words * sizeof(uint32_t) > (256ull << 20);
#define TNG_DECODE_LAUNCH(V, SC, GRID)                                                                          \
  hipLaunchKernelGGL((decode_vec_kernel<NORM, BITS, V, SC>), dim3((uint32_t)(GRID)), dim3(kBlock), 0, s, codes,  \
                     scales, reinterpret_cast<const float4*>(gref), reinterpret_cast<const float4*>(gref2),      \
                     reinterpret_cast<float4*>(vbar), reinterpret_cast<float4*>(w),                              \
                     reinterpret_cast<float4*>(ref_out), nvec, c.words, c.M, c.eps, inv_m, lr, c.means)
    if (big_tiles >= 2048) {
      if (stream_codes) {
        TNG_DECODE_LAUNCH(kDecodeLoads, true, big_tiles);
      } else {
        TNG_DECODE_LAUNCH(kDecodeLoads, false, big_tiles);
      }
    } else {  // few coordinates: small tiles so that every compute unit still gets work
      TNG_DECODE_LAUNCH(1, false, (nvec + kBlock - 1) / kBlock);
    }
#undef TNG_DECODE_LAUNCH
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess || dv == c.d) return e;
    hipLaunchKernelGGL((decode_scalar_kernel<NORM, BITS>), dim3(1), dim3(kBlock), 0, s, codes, scales, gref, gref2, vbar,
                       w, ref_out, dv, c.d, c.words, c.M, c.eps, inv_m, lr, c.means);  // the last d - dv < 16
    return hipGetLastError();
  }
  const uint64_t blocks = (c.d + kBlock - 1) / kBlock;
  hipLaunchKernelGGL((decode_scalar_kernel<NORM, BITS>), dim3((uint32_t)blocks), dim3(kBlock), 0, s, codes,
                     scales, gref, gref2, vbar, w, ref_out, (uint64_t)0, c.d, c.words, c.M, c.eps, inv_m, lr, c.means);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_fill_u32(uint32_t* p, uint64_t n, uint32_t value, hipStream_t s) {
  if (n == 0) return hipSuccess;
  const uint32_t gx = div_up_u32(n, kBlock);
  hipLaunchKernelGGL(fill_u32_kernel, dim3(gx < 8192u ? gx : 8192u), dim3(kBlock), 0, s, p, n, value);
  return hipGetLastError();
}

hipError_t launch_copy_f32(float* dst, const float* src, uint64_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  if (vec_ok(n, dst, src, nullptr)) {
    const uint32_t gx = div_up_u32(n / 4, (uint64_t)kBlock * kCopyPerThread);
    hipLaunchKernelGGL(copy_f32x4_kernel, dim3(gx < kMaxGridX ? gx : kMaxGridX), dim3(kBlock), 0, s,
                       reinterpret_cast<float4*>(dst), reinterpret_cast<const float4*>(src), n / 4);
  } else {
    const uint32_t gx = div_up_u32(n, kBlock);
    hipLaunchKernelGGL(copy_f32_kernel, dim3(gx < 16384u ? gx : 16384u), dim3(kBlock), 0, s, dst, src, n);
  }
  return hipGetLastError();
}

hipError_t launch_window_mean(const float* history, uint32_t window, uint32_t first, uint64_t d, float* out,
                              hipStream_t s) {
  if (vec_ok(d, history, out, nullptr)) {
    const uint32_t gx = div_up_u32(d / 4, kBlock);
    hipLaunchKernelGGL(window_mean_vec_kernel, dim3(gx < 16384u ? gx : 16384u), dim3(kBlock), 0, s,
                       reinterpret_cast<const float4*>(history), window, first, d / 4, 1.0f / (float)window,
                       reinterpret_cast<float4*>(out));
  } else {
    const uint32_t gx = div_up_u32(d, kBlock);
    hipLaunchKernelGGL(window_mean_kernel, dim3(gx < 16384u ? gx : 16384u), dim3(kBlock), 0, s, history, window, first,
                       d, 1.0f / (float)window, out);
  }
  return hipGetLastError();
}

hipError_t launch_rng_draws(uint32_t k0, uint32_t k1, uint32_t iter, uint32_t worker, uint32_t stream,
                            uint64_t first, uint64_t count, uint32_t* out, hipStream_t s) {
  if (count == 0) return hipSuccess;
  const uint32_t gx = div_up_u32(count, kBlock);
  hipLaunchKernelGGL(rng_draws_kernel, dim3(gx < 8192u ? gx : 8192u), dim3(kBlock), 0, s, k0, k1, iter,
                     worker, stream, first, count, out);
  return hipGetLastError();
}

hipError_t launch_absmax_finish(const float* partials, uint32_t nblocks, uint32_t M, float* scales, hipStream_t s) {
  hipLaunchKernelGGL(absmax_finish_kernel, dim3(M), dim3(kBlock), 0, s, partials, nblocks, M, scales);
  return hipGetLastError();
}

hipError_t launch_absmax(const CodecShape& c, const float* g, const float* gref, const float* gref2,
                         float* partials, float* scales, hipStream_t s) {
  switch (c.norm) {
    case kNormNone: return absmax_dispatch<kNormNone>(c, g, nullptr, nullptr, partials, scales, s);
    case kNormSub: return absmax_dispatch<kNormSub>(c, g, gref, nullptr, partials, scales, s);
    case kNormQuot: return absmax_dispatch<kNormQuot>(c, g, gref, nullptr, partials, scales, s);
    case kNormMean: return absmax_dispatch<kNormMean>(c, g, nullptr, nullptr, partials, scales, s);
    default: return absmax_dispatch<kNormComb>(c, g, gref, gref2, partials, scales, s);
  }
}

size_t tree_sum_scratch(uint64_t d, uint32_t M) {
  const uint64_t nchunks = (d + kTreeChunk - 1) / kTreeChunk;
  const uint64_t ngroups = (nchunks + kTreeGroup - 1) / kTreeGroup;
  return (size_t)((2 * nchunks + ngroups) * M);  // chunk sums, chunk (min, max) pairs, group sums
}

namespace {
template <int NORM, bool SQUARE, bool MINMAX>
hipError_t tree_sum_launch(const CodecShape& c, const float* g, const float* gref, const float* gref2, double* sums,
                           float* out, float* scales, hipStream_t s) {
  const uint64_t nchunks = (c.d + kTreeChunk - 1) / kTreeChunk;
  const uint64_t ngroups = (nchunks + kTreeGroup - 1) / kTreeGroup;
  float2* minmax = reinterpret_cast<float2*>(sums + nchunks * c.M);
  double* group_sums = sums + 2 * nchunks * c.M;
  const uint32_t gx = (uint32_t)((nchunks + kWavesPerBlock - 1) / kWavesPerBlock);
  constexpr bool kSharedRef = NORM == kNormSub || NORM == kNormQuot || NORM == kNormComb;
  const uint64_t whole = c.d / kTreeChunk;  // chunks that lie inside the rows entirely
  if (SQUARE && kSharedRef && whole != 0 && aligned16_or_null(gref, gref2)) {
    const uint32_t gw = (uint32_t)((whole + kWavesPerBlock - 1) / kWavesPerBlock);
    int mc = 4;  // workers per workgroup that share the reference tile in registers
    while (mc > 1 && (uint64_t)gw * ((c.M + mc - 1) / mc) < 2048) mc >>= 1;
    const GradRows rows{g, c.d};
    const float4* r4 = reinterpret_cast<const float4*>(gref);
    const float4* r24 = reinterpret_cast<const float4*>(gref2);
    dim3 grid(gw, (c.M + mc - 1) / mc);
    if (mc == 4) {
      hipLaunchKernelGGL((l2_chunk_kernel<kSharedRef ? NORM : kNormSub, 4>), grid, dim3(kBlock), 0, s, rows, r4, r24, sums,
                         whole, nchunks, c.eps, c.M);
    } else if (mc == 2) {
      hipLaunchKernelGGL((l2_chunk_kernel<kSharedRef ? NORM : kNormSub, 2>), grid, dim3(kBlock), 0, s, rows, r4, r24, sums,
                         whole, nchunks, c.eps, c.M);
    } else {
      hipLaunchKernelGGL((l2_chunk_kernel<kSharedRef ? NORM : kNormSub, 1>), grid, dim3(kBlock), 0, s, rows, r4, r24, sums,
                         whole, nchunks, c.eps, c.M);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (whole < nchunks) {  // the ragged last chunk of every row
      if (c.d % 4 == 0) {
        hipLaunchKernelGGL((tree_chunk_kernel<NORM, SQUARE, true, false>), dim3(1, c.M), dim3(kBlock), 0, s, g, gref,
                           gref2, c.means, sums, minmax, c.d, whole, nchunks, nchunks, c.eps, c.M, 1u);
      } else {
        hipLaunchKernelGGL((tree_chunk_kernel<NORM, SQUARE, false, false>), dim3(1, c.M), dim3(kBlock), 0, s, g, gref,
                           gref2, c.means, sums, minmax, c.d, whole, nchunks, nchunks, c.eps, c.M, 1u);
      }
      e = hipGetLastError();
      if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((tree_finish_kernel<false>), dim3(c.M), dim3(kBlock), 0, s, sums, group_sums, nullptr, nchunks,
                       ngroups, c.d, out, scales);
    return hipGetLastError();
  }
  // workers per workgroup: as many as leave 2048 workgroups (only worth it when a reference is shared)
  uint32_t wpb = 1;
  if (SQUARE && gref != nullptr)
    while (wpb < 8 && wpb < c.M && (uint64_t)gx * ((c.M + 2 * wpb - 1) / (2 * wpb)) >= 2048) wpb *= 2;
  dim3 grid(gx, (c.M + wpb - 1) / wpb);
  if (aligned16_or_null(gref, gref2)) {
    // the last chunk of rows whose length is not a multiple of 4 goes element by element
    const uint64_t vec_end = c.d % 4 == 0 ? nchunks : whole;
    if (vec_end != 0)
      hipLaunchKernelGGL((tree_chunk_kernel<NORM, SQUARE, true, MINMAX>), grid, dim3(kBlock), 0, s, g, gref, gref2,
                         c.means, sums, minmax, c.d, (uint64_t)0, vec_end, nchunks, c.eps, c.M, wpb);
    if (vec_end != nchunks)
      hipLaunchKernelGGL((tree_chunk_kernel<NORM, SQUARE, false, MINMAX>), dim3(1, c.M), dim3(kBlock), 0, s, g, gref,
                         gref2, c.means, sums, minmax, c.d, vec_end, nchunks, nchunks, c.eps, c.M, 1u);
  } else {
    hipLaunchKernelGGL((tree_chunk_kernel<NORM, SQUARE, false, MINMAX>), grid, dim3(kBlock), 0, s, g, gref, gref2,
                       c.means, sums, minmax, c.d, (uint64_t)0, nchunks, nchunks, c.eps, c.M, wpb);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((tree_finish_kernel<!SQUARE>), dim3(c.M), dim3(kBlock), 0, s, sums, group_sums,
                     MINMAX ? minmax : nullptr, nchunks, ngroups, c.d, out, scales);
  return hipGetLastError();
}
}  // namespace

hipError_t launch_worker_means(const CodecShape& c, const float* g, double* sums, float* means, float* scales,
                               hipStream_t s) {
  if (scales != nullptr) return tree_sum_launch<kNormNone, false, true>(c, g, nullptr, nullptr, sums, means, scales, s);
  return tree_sum_launch<kNormNone, false, false>(c, g, nullptr, nullptr, sums, means, nullptr, s);
}

hipError_t launch_l2_scales(const CodecShape& c, const float* g, const float* gref, const float* gref2, double* sums,
                            float* scales, hipStream_t s) {
  switch (c.norm) {
    case kNormNone: return tree_sum_launch<kNormNone, true, false>(c, g, nullptr, nullptr, sums, scales, nullptr, s);
    case kNormSub: return tree_sum_launch<kNormSub, true, false>(c, g, gref, nullptr, sums, scales, nullptr, s);
    case kNormQuot: return tree_sum_launch<kNormQuot, true, false>(c, g, gref, nullptr, sums, scales, nullptr, s);
    case kNormMean: return tree_sum_launch<kNormMean, true, false>(c, g, nullptr, nullptr, sums, scales, nullptr, s);
    default: return tree_sum_launch<kNormComb, true, false>(c, g, gref, gref2, sums, scales, nullptr, s);
  }
}

size_t candidate_scratch_bytes(const CodecShape& c) {
  // 2-bit codes, largest-magnitude scale, a shared reference or none, whole wavefront tiles, and enough
  // elements (2^26: 256 MiB of gradients) for the extra launches of the sample to be noise
  // (not the quotient forms: there |v| is near 1 everywhere and a third of the elements code non-zero)
  if (c.bits != 2 || c.scale_l2 != 0 || (c.norm != kNormNone && c.norm != kNormSub) || c.d % 1024 != 0) return 0;
  if ((uint64_t)c.M * c.d < (1ull << 26) || c.d / 1024 < 4 * (uint64_t)kSampleStride) return 0;
  return candidate_head_bytes(c.M) + (size_t)c.M * (c.d / 1024) * kSlotEntries * sizeof(uint32_t);
}

bool candidates_apply(const CodecShape& c, const float* g, const float* gref, const float* gref2,
                      const uint32_t* codes) {
  return candidate_scratch_bytes(c) != 0 && aligned16_or_null(g, gref, gref2, codes);
}

hipError_t launch_absmax_candidates(const CodecShape& c, uint32_t iter, const float* g, const float* gref,
                                    const float* gref2, float* partials, void* scratch, float* scales, hipStream_t s) {
  const CandidateScratch cs = candidate_scratch(c, scratch);
  if (c.norm == kNormSub) return absmax_candidates_dispatch<kNormSub>(c, iter, g, gref, nullptr, partials, cs, scales, s);
  return absmax_candidates_dispatch<kNormNone>(c, iter, g, nullptr, nullptr, partials, cs, scales, s);
}

hipError_t launch_quantize_candidates(const CodecShape& c, uint32_t iter, const float* g, const float* gref,
                                      const float* gref2, const float* scales, void* scratch, uint32_t* codes,
                                      hipStream_t s) {
  const CandidateScratch cs = candidate_scratch(c, scratch);
  if (c.norm == kNormSub) return quantize_candidates_dispatch<kNormSub>(c, iter, g, gref, nullptr, scales, cs, codes, s);
  return quantize_candidates_dispatch<kNormNone>(c, iter, g, nullptr, nullptr, scales, cs, codes, s);
}

hipError_t launch_quantize_pack(const CodecShape& c, uint32_t iter, const float* g, const float* gref,
                                const float* gref2, float* scales, uint32_t* codes, const float* partials,
                                uint32_t fused_rows, hipStream_t s) {
#define TNG_Q(NORM, R1, R2)                                                                                      \
  return c.bits == 2 ? quantize_dispatch<NORM, 2>(c, iter, g, R1, R2, scales, codes, partials, fused_rows, s)    \
                     : quantize_dispatch<NORM, 4>(c, iter, g, R1, R2, scales, codes, partials, fused_rows, s)
  switch (c.norm) {
    case kNormNone: TNG_Q(kNormNone, nullptr, nullptr);
    case kNormSub: TNG_Q(kNormSub, gref, nullptr);
    case kNormQuot: TNG_Q(kNormQuot, gref, nullptr);
    case kNormMean: TNG_Q(kNormMean, nullptr, nullptr);
    default: TNG_Q(kNormComb, gref, gref2);
  }
#undef TNG_Q
}

namespace {
template <int NORM, int BITS>
hipError_t single_pass_dispatch(const CodecShape& c, uint32_t iter, const float* g, const float* gref,
                                const float* gref2, float* scales, uint32_t* codes, bool decode, float* vbar,
                                float* w, float lr, float* ref_out, hipStream_t s) {
#define TNG_SP(MC, DEC)                                                                                             \
  hipLaunchKernelGGL((single_pass_kernel<NORM, BITS, MC, DEC>), dim3(1), dim3(kBlock), 0, s, GradRows{g, c.d},       \
                     reinterpret_cast<const float4*>(gref), reinterpret_cast<const float4*>(gref2), scales, codes,   \
                     c.d / 4, c.words, c.M, c.eps, c.k0, c.k1, iter, reinterpret_cast<float4*>(vbar),                \
                     reinterpret_cast<float4*>(w), reinterpret_cast<float4*>(ref_out), 1.0f / (float)c.M, lr)
  if (c.M <= 8) {
    if (decode) {
      TNG_SP(8, true);
    } else {
      TNG_SP(8, false);
    }
  } else if (decode) {
    TNG_SP(16, true);
  } else {
    TNG_SP(16, false);
  }
#undef TNG_SP
  return hipGetLastError();
}
}  // namespace

bool single_pass_applies(const CodecShape& c, const float* g, const float* gref, const float* gref2, const float* vbar,
                         const float* w, const float* ref_out) {
  return c.scale_l2 == 0 && c.norm != kNormMean && c.d % 4 == 0 && c.d <= 4 * (uint64_t)kBlock &&
         c.M <= (uint32_t)kSinglePassMaxWorkers && aligned16_or_null(g, gref, gref2) &&
         aligned16_or_null(vbar, w, ref_out);
}

hipError_t launch_single_pass(const CodecShape& c, uint32_t iter, const float* g, const float* gref, const float* gref2,
                              float* scales, uint32_t* codes, bool decode, float* vbar, float* w, float lr,
                              float* ref_out, hipStream_t s) {
  if (!single_pass_applies(c, g, gref, gref2, vbar, w, ref_out)) return hipErrorInvalidValue;
#define TNG_SPD(NORM, R1, R2)                                                                                        \
  return c.bits == 2 ? single_pass_dispatch<NORM, 2>(c, iter, g, R1, R2, scales, codes, decode, vbar, w, lr, ref_out, s) \
                     : single_pass_dispatch<NORM, 4>(c, iter, g, R1, R2, scales, codes, decode, vbar, w, lr, ref_out, s)
  switch (c.norm) {
    case kNormNone: TNG_SPD(kNormNone, nullptr, nullptr);
    case kNormSub: TNG_SPD(kNormSub, gref, nullptr);
    case kNormQuot: TNG_SPD(kNormQuot, gref, nullptr);
    default: TNG_SPD(kNormComb, gref, gref2);
  }
#undef TNG_SPD
}

hipError_t launch_decode(const CodecShape& c, const uint32_t* codes, const float* scales, const float* gref,
                         const float* gref2, float* vbar, float* w, float lr, float* ref_out, hipStream_t s) {
#define TNG_D(NORM, R1, R2)                                                                          \
  return c.bits == 2 ? decode_dispatch<NORM, 2>(c, codes, scales, R1, R2, vbar, w, lr, ref_out, s)   \
                     : decode_dispatch<NORM, 4>(c, codes, scales, R1, R2, vbar, w, lr, ref_out, s)
  switch (c.norm) {
    case kNormNone: TNG_D(kNormNone, nullptr, nullptr);
    case kNormSub: TNG_D(kNormSub, gref, nullptr);
    case kNormQuot: TNG_D(kNormQuot, gref, nullptr);
    case kNormMean: TNG_D(kNormMean, nullptr, nullptr);
    default: TNG_D(kNormComb, gref, gref2);
  }
#undef TNG_D
}

}  // namespace tng
