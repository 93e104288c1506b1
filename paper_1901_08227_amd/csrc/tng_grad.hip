// Local-gradient kernels of libtng (Algorithm 1: "each server calculates local gradient"), gfx950.
//
// Logistic regression is two matrix-vector products per worker (z = X_B w, g = X_B^T r) with a
// different X_B per worker and a single vector on the other side, so there is no dense
// matrix-matrix contraction to put on the matrix cores: both passes stream the minibatch rows
// with coalesced 16-byte loads and are bound by HBM bandwidth.  Gradients are compared with a
// tolerance, so these kernels use fused multiply-adds explicitly; the Rosenbrock gradient keeps a
// fixed expression tree without them and is reproducible bit for bit.
#include "tng_device.hpp"
#include "tng_kernels.hpp"

#include <mutex>

namespace tng {

namespace {

constexpr int kWavesPerBlock = kBlock / kWave;

// Background: index "uniformly sampled" -- idx = (draw * n_rows) >> 32, draws from stream 1.
__device__ __forceinline__ uint32_t minibatch_row(uint32_t k0, uint32_t k1, uint32_t iter, uint32_t m, uint32_t j,
                                                  uint64_t n_rows) {
  const U32x4 r = philox4x32_10(j >> 2, m, iter, 1u, k0, k1);
  const uint32_t lane = j & 3u;
  const uint32_t x = lane == 0 ? r.x : lane == 1 ? r.y : lane == 2 ? r.z : r.w;
  return (uint32_t)(((uint64_t)x * n_rows) >> 32);
}

__global__ __launch_bounds__(kBlock) void minibatch_indices_kernel(uint32_t k0, uint32_t k1, uint32_t iter,
                                                                   uint32_t batch,
                                                                   const uint64_t* __restrict__ n_rows,
                                                                   uint32_t* __restrict__ idx) {
  const uint32_t m = blockIdx.y;
  const uint32_t j = blockIdx.x * kBlock + threadIdx.x;
  if (j >= batch) return;
  idx[(uint64_t)m * batch + j] = minibatch_row(k0, k1, iter, m, j, n_rows[m]);
}

__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  if (lane == 0) red[wave] = v;
  __syncthreads();
  float s = red[0];
#pragma unroll
  for (int k = 1; k < kWavesPerBlock; ++k) s += red[k];
  return s;
}

// Maximum over the workgroup (any size up to 1024 threads); valid in thread 0.  red: 16 floats of LDS.
__device__ __forceinline__ float block_max(float v, float* red) {
  v = wave_max(v);
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  __syncthreads();  // red may still be read from an earlier call
  if (lane == 0) red[wave] = v;
  __syncthreads();
  const int nw = (blockDim.x + kWave - 1) / kWave;
  float r = red[0];
  for (int k = 1; k < nw; ++k) r = fmaxf(r, red[k]);
  return r;
}

// Largest |normalize(g)| over the four components of a float4 of gradient values (fused scale pass).
__device__ __forceinline__ float absmax4(const ScaleFusion& f, const float4& g, const float4& r1, const float4& r2) {
  return fmaxf(fmaxf(fabsf(normalize_dyn(f.norm, g.x, r1.x, r2.x, f.eps)), fabsf(normalize_dyn(f.norm, g.y, r1.y, r2.y, f.eps))),
               fmaxf(fabsf(normalize_dyn(f.norm, g.z, r1.z, r2.z, f.eps)), fabsf(normalize_dyn(f.norm, g.w, r1.w, r2.w, f.eps))));
}

__device__ __forceinline__ void load_refs4(const ScaleFusion& f, uint64_t q, float4& r1, float4& r2) {
  r1 = make_float4(0.f, 0.f, 0.f, 0.f);
  r2 = make_float4(1.f, 1.f, 1.f, 1.f);
  if (f.norm != kNormNone) r1 = reinterpret_cast<const float4*>(f.gref)[q];
  if (f.norm == kNormComb) r2 = reinterpret_cast<const float4*>(f.gref2)[q];
}

// The same two helpers with the kind of normalisation known at compile time: no branch around the loads,
// so the compiler can count them (see the pipelined CSR gradient kernel).
template <int NORM>
__device__ __forceinline__ void load_refs4_t(const ScaleFusion& f, uint64_t q, float4& r1, float4& r2) {
  r1 = make_float4(0.f, 0.f, 0.f, 0.f);
  r2 = make_float4(1.f, 1.f, 1.f, 1.f);
  if (NORM != kNormNone) r1 = reinterpret_cast<const float4*>(f.gref)[q];
  if (NORM == kNormComb) r2 = reinterpret_cast<const float4*>(f.gref2)[q];
}

template <int NORM>
__device__ __forceinline__ float absmax4_t(const ScaleFusion& f, const float4& g, const float4& r1, const float4& r2) {
  return fmaxf(fmaxf(fabsf(normalize_dyn(NORM, g.x, r1.x, r2.x, f.eps)), fabsf(normalize_dyn(NORM, g.y, r1.y, r2.y, f.eps))),
               fmaxf(fabsf(normalize_dyn(NORM, g.z, r1.z, r2.z, f.eps)), fabsf(normalize_dyn(NORM, g.w, r1.w, r2.w, f.eps))));
}

// sigma(z) - y without cancellation for the labels 0 and 1.
__device__ __forceinline__ float logistic_residual(float z, float y) {
  const float e = expf(-fabsf(z));           // in (0, 1]
  const float small = e / (1.0f + e);          // sigma(-|z|)
  const float big = 1.0f / (1.0f + e);         // sigma(|z|)
  const float sig = z >= 0.f ? big : small;
  if (y == 1.0f) return z >= 0.f ? -small : -big;  // sigma(z) - 1 = -sigma(-z)
  if (y == 0.0f) return sig;
  return sig - y;
}

// z_i = x_i . w and r_i = sigma(z_i) - y_i for ROWS minibatch rows per workgroup (w is fetched once
// for all of them; each row keeps the accumulation order it has with ROWS = 1).
template <bool VEC, int ROWS>
__global__ __launch_bounds__(kBlock) void logreg_dense_resid_kernel(const float* const* __restrict__ Xs,
                                                                    const float* const* __restrict__ ys,
                                                                    const uint64_t* __restrict__ n_rows,
                                                                    uint32_t* __restrict__ idx,
                                                                    const float* __restrict__ w,
                                                                    float* __restrict__ resid, uint64_t d,
                                                                    uint32_t batch, uint32_t k0, uint32_t k1,
                                                                    uint32_t iter) {
  __shared__ float red[kWavesPerBlock];
  const uint32_t m = blockIdx.y, i0 = blockIdx.x * ROWS;
  // the row ids are drawn here (one launch fewer) and left in idx for the accumulation pass
  uint32_t row[ROWS];
  GlobalPtr<float> x[ROWS];
#pragma unroll
  for (int r = 0; r < ROWS; ++r) {
    row[r] = minibatch_row(k0, k1, iter, m, min(i0 + r, batch - 1), n_rows[m]);  // a short last group repeats its last row
    if (threadIdx.x == 0 && i0 + r < batch) idx[(uint64_t)m * batch + i0 + r] = row[r];
    x[r] = as_global(Xs[m]) + (uint64_t)row[r] * d;
  }
  float acc[ROWS];
  if (VEC) {
    const float4* w4 = reinterpret_cast<const float4*>(w);
    const uint64_t nvec = d / 4;
    float a0[ROWS], a1[ROWS], a2[ROWS], a3[ROWS];
#pragma unroll
    for (int r = 0; r < ROWS; ++r) a0[r] = a1[r] = a2[r] = a3[r] = 0.f;
#pragma unroll 8 / ROWS
    for (uint64_t k = threadIdx.x; k < nvec; k += kBlock) {
      const float4 wv = w4[k];
#pragma unroll
      for (int r = 0; r < ROWS; ++r) {
        const float4 xv = load4_stream_any(x[r], k);
        a0[r] = __builtin_fmaf(xv.x, wv.x, a0[r]);
        a1[r] = __builtin_fmaf(xv.y, wv.y, a1[r]);
        a2[r] = __builtin_fmaf(xv.z, wv.z, a2[r]);
        a3[r] = __builtin_fmaf(xv.w, wv.w, a3[r]);
      }
    }
    if (4 * nvec + threadIdx.x < d) {  // the last d mod 4 columns
      const uint64_t k = 4 * nvec + threadIdx.x;
      const float wk = w[k];
#pragma unroll
      for (int r = 0; r < ROWS; ++r) a0[r] = __builtin_fmaf(x[r][k], wk, a0[r]);
    }
#pragma unroll
    for (int r = 0; r < ROWS; ++r) acc[r] = (a0[r] + a1[r]) + (a2[r] + a3[r]);
  } else {
#pragma unroll
    for (int r = 0; r < ROWS; ++r) acc[r] = 0.f;
    for (uint64_t k = threadIdx.x; k < d; k += kBlock) {
      const float wk = w[k];
#pragma unroll
      for (int r = 0; r < ROWS; ++r) acc[r] = __builtin_fmaf(x[r][k], wk, acc[r]);
    }
  }
#pragma unroll
  for (int r = 0; r < ROWS; ++r) {
    if (r > 0) __syncthreads();  // red is reused
    const float z = block_sum(acc[r], red);
    if (threadIdx.x == 0 && i0 + r < batch)
      resid[(uint64_t)m * batch + i0 + r] = logistic_residual(z, as_global(ys[m])[row[r]]);
  }
}

// g_m[k] = (1/B) sum_i r_i X[idx_i][k] + l2 w[k]; a thread owns 4 (VEC) or 1 columns.
template <bool VEC, bool FUSE>
__global__ __launch_bounds__(kBlock) void logreg_dense_grad_kernel(const float* const* __restrict__ Xs,
                                                                   const uint32_t* __restrict__ idx,
                                                                   const float* __restrict__ resid,
                                                                   const float* __restrict__ w,
                                                                   float* __restrict__ g, uint64_t d,
                                                                   uint64_t first_col, uint32_t batch, float inv_b,
                                                                   float l2, ScaleFusion fuse) {
  __shared__ float sR[kBlock];
  __shared__ uint32_t sRow[kBlock];
  __shared__ float red[16];
  const uint32_t m = blockIdx.y;
  const GlobalPtr<float> X = as_global(Xs[m]);
  const uint64_t col = first_col + (uint64_t)blockIdx.x * kBlock + threadIdx.x;  // float4 (VEC) or float index
  const uint64_t ncol = VEC ? d / 4 : d;
  const bool active = col < ncol;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (uint32_t base = 0; base < batch; base += kBlock) {
    __syncthreads();
    if (base + threadIdx.x < batch) {
      sR[threadIdx.x] = resid[(uint64_t)m * batch + base + threadIdx.x];
      sRow[threadIdx.x] = idx[(uint64_t)m * batch + base + threadIdx.x];
    }
    __syncthreads();
    if (active) {
      const uint32_t cnt = min((uint32_t)kBlock, batch - base);
      if (VEC) {
#pragma unroll 8
        for (uint32_t i = 0; i < cnt; ++i) {
          const float4 xv = load4_stream_any(X + (uint64_t)sRow[i] * d, col);
          const float r = sR[i];
          acc.x = __builtin_fmaf(r, xv.x, acc.x);
          acc.y = __builtin_fmaf(r, xv.y, acc.y);
          acc.z = __builtin_fmaf(r, xv.z, acc.z);
          acc.w = __builtin_fmaf(r, xv.w, acc.w);
        }
      } else {
#pragma unroll 8
        for (uint32_t i = 0; i < cnt; ++i) acc.x = __builtin_fmaf(sR[i], X[(uint64_t)sRow[i] * d + col], acc.x);
      }
    }
  }
  float amax = 0.f;
  if (active) {
    if (VEC) {
      const float4 wv = reinterpret_cast<const float4*>(w)[col];
      float4 o;
      o.x = __builtin_fmaf(l2, wv.x, acc.x * inv_b);
      o.y = __builtin_fmaf(l2, wv.y, acc.y * inv_b);
      o.z = __builtin_fmaf(l2, wv.z, acc.z * inv_b);
      o.w = __builtin_fmaf(l2, wv.w, acc.w * inv_b);
      store4_any(g + (uint64_t)m * d, col, o);
      if (FUSE) {
        float4 r1, r2;
        load_refs4(fuse, col, r1, r2);
        amax = absmax4(fuse, o, r1, r2);
      }
    } else {
      g[(uint64_t)m * d + col] = __builtin_fmaf(l2, w[col], acc.x * inv_b);
    }
  }
  if (FUSE) {
    amax = block_max(amax, red);
    if (threadIdx.x == 0) fuse.partials[(uint64_t)blockIdx.x * gridDim.y + m] = amax;
  }
}

// The same for problems with few columns (a handful of workgroups in all): 1024 threads, COLS float4
// columns times RG row groups; the minibatch rows are dealt round-robin to the row groups, which run
// side by side, and their partial sums are added in the fixed order ((p0 + p1) + p2) + ...  Cuts the
// chain of dependent row fetches to 1/RG; narrow column blocks (32 x 32) also spread a tiny problem
// over eight times as many compute units, each of which can only pull so many bytes per microsecond.
constexpr int kSplitThreads = 1024;
template <int COLS, bool FUSE>
__global__ __launch_bounds__(kSplitThreads) void logreg_dense_grad_split_kernel(
    const float* const* __restrict__ Xs, const uint32_t* __restrict__ idx, const float* __restrict__ resid,
    const float* __restrict__ w, float* __restrict__ g, uint64_t d, uint32_t batch, float inv_b, float l2,
    ScaleFusion fuse) {
  constexpr int RG = kSplitThreads / COLS;
  __shared__ float sR[kBlock];
  __shared__ uint32_t sRow[kBlock];
  __shared__ float4 sAcc[RG - 1][COLS];
  __shared__ float red[16];
  const uint32_t m = blockIdx.y;
  const uint32_t tx = threadIdx.x % COLS, rg = threadIdx.x / COLS;
  const GlobalPtr<float> X = as_global(Xs[m]);
  const uint64_t col = (uint64_t)blockIdx.x * COLS + tx;  // float4 index
  const bool active = col < d / 4;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (uint32_t base = 0; base < batch; base += kBlock) {
    __syncthreads();
    if (threadIdx.x < (uint32_t)kBlock && base + threadIdx.x < batch) {
      sR[threadIdx.x] = resid[(uint64_t)m * batch + base + threadIdx.x];
      sRow[threadIdx.x] = idx[(uint64_t)m * batch + base + threadIdx.x];
    }
    __syncthreads();
    if (active) {
      const uint32_t cnt = min((uint32_t)kBlock, batch - base);
#pragma unroll 8
      for (uint32_t i = rg; i < cnt; i += RG) {
        const float4 xv = load4_stream(X + (uint64_t)sRow[i] * d, col);
        const float r = sR[i];
        acc.x = __builtin_fmaf(r, xv.x, acc.x);
        acc.y = __builtin_fmaf(r, xv.y, acc.y);
        acc.z = __builtin_fmaf(r, xv.z, acc.z);
        acc.w = __builtin_fmaf(r, xv.w, acc.w);
      }
    }
  }
  if (rg > 0) sAcc[rg - 1][tx] = acc;
  __syncthreads();
  float amax = 0.f;
  if (active && rg == 0) {
#pragma unroll
    for (int k = 0; k < RG - 1; ++k) {
      const float4 p = sAcc[k][tx];
      acc.x = acc.x + p.x;
      acc.y = acc.y + p.y;
      acc.z = acc.z + p.z;
      acc.w = acc.w + p.w;
    }
    const float4 wv = reinterpret_cast<const float4*>(w)[col];
    float4 o;
    o.x = __builtin_fmaf(l2, wv.x, acc.x * inv_b);
    o.y = __builtin_fmaf(l2, wv.y, acc.y * inv_b);
    o.z = __builtin_fmaf(l2, wv.z, acc.z * inv_b);
    o.w = __builtin_fmaf(l2, wv.w, acc.w * inv_b);
    reinterpret_cast<float4*>(g + (uint64_t)m * d)[col] = o;
    if (FUSE) {
      float4 r1, r2;
      load_refs4(fuse, col, r1, r2);
      amax = absmax4(fuse, o, r1, r2);
    }
  }
  if (FUSE) {
    amax = block_max(amax, red);
    if (threadIdx.x == 0) fuse.partials[(uint64_t)blockIdx.x * gridDim.y + m] = amax;
  }
}

// One pass over the minibatch rows for wide dense problems (4096 <= d / 4 <= 16384 float4 columns): a
// workgroup takes whole rows, one at a time, and KEEPS the row on chip between the two uses it has -- the
// dot product z = x . w, and, once sigma(z) - y is known, the accumulation r x into the workgroup's
// partial gradient -- so that X_B is read from memory once instead of twice (the separate residual and
// accumulation passes each stream it at 6.2 TB/s, which is all the memory system gives; re-reading a
// block right after it was read, out of the 256 MB last-level cache, measured no faster than HBM).
// A row of up to 256 KiB fits neither store alone: each of the 512 threads (one workgroup per compute
// unit, so 256 registers per thread) parks NL = min(NV, 16) float4 of the row in LDS (128 KiB per
// workgroup; a thread reads back only what it wrote) and holds the other NV - NL in registers, next to its
// NV float4 of partial gradient.  The LDS half is loaded from memory straight into LDS, so that the whole
// row is requested at once.
// The workgroups of a worker split its minibatch rows; their partial gradients go to scratch
// parts[m][s][d] and logreg_dense_parts_kernel adds them in workgroup order.
constexpr int kRowsThreads = 512;
constexpr int kRowsWaves = kRowsThreads / kWave;
// 16 bytes per lane from memory straight into LDS: lane l of the wavefront writes the l-th 16 bytes behind
// dst, which is the same for the whole wavefront; counted by vmcnt like any load.  Non-temporal (policy bit
// 2): the row is read once.  (The builtin exists in the device pass only.)
constexpr int kRowsStagger = 55;  // s_sleep units of 64 clocks: about 1.7 microseconds
typedef __attribute__((address_space(3))) void* LdsPtr;
__device__ __forceinline__ void load16_to_lds(GlobalPtr<v4f_t> src, LdsPtr dst) {
#if defined(__HIP_DEVICE_COMPILE__)
  __builtin_amdgcn_global_load_lds(src, dst, 16, 0, 2);
#endif
}
constexpr int kRowsLds = 16;  // float4 per thread kept in LDS
template <int NV, bool FULL>
__global__ __launch_bounds__(kRowsThreads) void logreg_dense_rows_kernel(const float* const* __restrict__ Xs,
                                                                         const float* const* __restrict__ ys,
                                                                         const uint64_t* __restrict__ n_rows,
                                                                         uint32_t* __restrict__ idx,
                                                                         const float* __restrict__ w,
                                                                         float* __restrict__ parts, uint64_t d,
                                                                         uint32_t batch, uint32_t k0, uint32_t k1,
                                                                         uint32_t iter) {
  constexpr int NL = NV < kRowsLds ? NV : kRowsLds;
  constexpr int NR = NV - NL;
  constexpr int TR = 4;                // float4 of the LDS half read back at a time when the row is added
  constexpr int TW = NV < 8 ? NV : 8;  // float4 of w on their way at a time
  static_assert(NL % TR == 0 && NL % TW == 0 && NR % TW == 0, "both halves are worked through in whole batches");
  constexpr int kWaitVmem = 0x0F70;         // s_waitcnt vmcnt(0)
  constexpr int kWaitLds = 0xC07F;          // s_waitcnt lgkmcnt(0)
  extern __shared__ float4 rowl[];  // [NL][kRowsThreads]
  __shared__ float red[2][kRowsWaves];
  const uint32_t m = blockIdx.y, s = blockIdx.x, S = gridDim.x, t = threadIdx.x;
  const uint32_t wave_first = (uint32_t)__builtin_amdgcn_readfirstlane((int)(t / kWave)) * kWave;  // a scalar
  const uint32_t nvec = (uint32_t)(d / 4);
  const GlobalPtr<float> X = as_global(Xs[m]);
  const GlobalPtr<float> y = as_global(ys[m]);
  const uint64_t n = n_rows[m];
  const float4* __restrict__ w4 = reinterpret_cast<const float4*>(w);
  // float4 column k of the thread: LDS half first (k < NL), register half after; clamped so that every load
  // is unconditional (FULL: d / 4 = NV * 512, nothing to clamp or mask)
  // (the thread index goes through an opaque copy per use site: otherwise the compiler computes all NV
  // column addresses of x and of w once, ahead of the row loop, and keeps them in 3 NV registers)
  auto opaque_t = [&]() {
    uint32_t v = t;
    asm volatile("" : "+v"(v));
    return v;
  };
  auto column_of = [&](uint32_t tt, int k) {
    return FULL ? tt + (uint32_t)k * kRowsThreads : min(tt + (uint32_t)k * kRowsThreads, nvec - 1);
  };
  auto column = [&](int k) { return column_of(t, k); };
  auto live = [&](int k) { return FULL || t + (uint32_t)k * kRowsThreads < nvec; };
  const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
  float4 acc[NV];
#pragma unroll
  for (int k = 0; k < NV; ++k) acc[k] = zero4;
  // A row is fetched (memory busy, arithmetic idle) and then worked on (the reverse), and workgroups that start
  // together stay in step: every compute unit fetches at once and the memory system idles while all of them
  // compute.  A quarter of the workgroups therefore starts at once and the others 1.7, 3.4 and 5.1 microseconds
  // later (about the length of the arithmetic on a row), so that the fetches of some fall into the arithmetic of
  // the others.  Measured at d = 2^16, M = 16, B = 256: iteration 0.236 -> 0.224 ms, this kernel 200
  // microseconds (with twice the delay 0.230 ms; with eight steps of 0.7 microseconds 204 microseconds).
  for (uint32_t q = (blockIdx.x + blockIdx.y * gridDim.x) % 4u; q > 0; --q) __builtin_amdgcn_s_sleep(kRowsStagger);
  uint32_t parity = 0;
  for (uint32_t i = s; i < batch; i += S, parity ^= 1u) {
    const uint32_t row = minibatch_row(k0, k1, iter, m, i, n);
    if (t == 0) idx[(uint64_t)m * batch + i] = row;
    const GlobalPtr<float> x = X + (uint64_t)row * d;
    // Requests of a row, in the order in which they come back: the first batch of w (out of the caches), the
    // register half, then the LDS half, which goes from memory straight into LDS (16 bytes per lane, lane l of
    // a wavefront to the l-th float4 behind the wavefront's address: each thread's own slot) -- so the whole
    // row, 256 KiB at d = 2^16, is in flight at once and no register carries the LDS half.
    float4 wa[TW];
    {
      const uint32_t tt = opaque_t();
#pragma unroll
      for (int k = 0; k < TW; ++k) wa[k] = w4[column_of(tt, k)];
    }
    float4 xr[NR > 0 ? NR : 1];
    {
      const uint32_t tt = opaque_t();
#pragma unroll
      for (int k = 0; k < NR; ++k) xr[k] = load4_stream(x, column_of(tt, NL + k));
    }
    {
      const uint32_t tt = opaque_t();
#pragma unroll
      for (int k = 0; k < NL; ++k)
        load16_to_lds(reinterpret_cast<GlobalPtr<v4f_t>>(x) + column_of(tt, k),
                      (LdsPtr)(rowl + k * kRowsThreads + wave_first));
    }
    __builtin_amdgcn_s_waitcnt(kWaitVmem);  // everything requested above has arrived, the LDS half in LDS
    asm volatile("" ::: "memory");
    float z0 = 0.f, z1 = 0.f, z2 = 0.f, z3 = 0.f;
#pragma unroll
    for (int k0b = 0; k0b < NL; k0b += TW) {
      if (k0b > 0) {
        const uint32_t tt = opaque_t();
#pragma unroll
        for (int k = 0; k < TW; ++k) wa[k] = w4[column_of(tt, k0b + k)];
      }
      const uint32_t tt = opaque_t();
#pragma unroll
      for (int k = 0; k < TW; ++k) {
        const float4 xl = rowl[(k0b + k) * kRowsThreads + tt];
        const float4 xv = live(k0b + k) ? xl : zero4;
        z0 = __builtin_fmaf(xv.x, wa[k].x, z0);
        z1 = __builtin_fmaf(xv.y, wa[k].y, z1);
        z2 = __builtin_fmaf(xv.z, wa[k].z, z2);
        z3 = __builtin_fmaf(xv.w, wa[k].w, z3);
      }
      asm volatile("" ::: "memory");  // keeps the next batch's loads behind this batch's use: registers are the scarce thing here
    }
#pragma unroll
    for (int k0b = 0; k0b < NR; k0b += TW) {
      const uint32_t tt = opaque_t();
#pragma unroll
      for (int k = 0; k < TW; ++k) wa[k] = w4[column_of(tt, NL + k0b + k)];
#pragma unroll
      for (int k = 0; k < TW; ++k) {
        if (!live(NL + k0b + k)) xr[k0b + k] = zero4;
        z0 = __builtin_fmaf(xr[k0b + k].x, wa[k].x, z0);
        z1 = __builtin_fmaf(xr[k0b + k].y, wa[k].y, z1);
        z2 = __builtin_fmaf(xr[k0b + k].z, wa[k].z, z2);
        z3 = __builtin_fmaf(xr[k0b + k].w, wa[k].w, z3);
      }
      asm volatile("" ::: "memory");
    }
    // z over the workgroup (two sets of slots alternate, so that one barrier per row is enough)
    const float zw = wave_sum((z0 + z1) + (z2 + z3));
    if (t % kWave == 0) red[parity][t / kWave] = zw;
    __syncthreads();
    float z = red[parity][0];
#pragma unroll
    for (int k = 1; k < kRowsWaves; ++k) z += red[parity][k];
    const float r = logistic_residual(z, y[row]);
#pragma unroll
    for (int k = 0; k < NR; ++k) {
      acc[NL + k].x = __builtin_fmaf(r, xr[k].x, acc[NL + k].x);
      acc[NL + k].y = __builtin_fmaf(r, xr[k].y, acc[NL + k].y);
      acc[NL + k].z = __builtin_fmaf(r, xr[k].z, acc[NL + k].z);
      acc[NL + k].w = __builtin_fmaf(r, xr[k].w, acc[NL + k].w);
    }
#pragma unroll
    for (int k0b = 0; k0b < NL; k0b += TR) {
      const uint32_t tt = opaque_t();
#pragma unroll
      for (int k = k0b; k < k0b + TR; ++k) {
        const float4 xl = rowl[k * kRowsThreads + tt];
        const float4 xv = live(k) ? xl : zero4;
        acc[k].x = __builtin_fmaf(r, xv.x, acc[k].x);
        acc[k].y = __builtin_fmaf(r, xv.y, acc[k].y);
        acc[k].z = __builtin_fmaf(r, xv.z, acc[k].z);
        acc[k].w = __builtin_fmaf(r, xv.w, acc[k].w);
      }
      asm volatile("" ::: "memory");
    }
    __builtin_amdgcn_s_waitcnt(kWaitLds);  // this row's LDS reads are done before the next row's loads write there
    asm volatile("" ::: "memory");
  }
  float4* __restrict__ out = reinterpret_cast<float4*>(parts + ((uint64_t)m * S + s) * d);
#pragma unroll
  for (int k = 0; k < NV; ++k)
    if (live(k)) store_stream(out + column(k), acc[k]);
}

// g_m = (1/B) (sum over the S partial gradients of worker m, in order) + l2 w; FUSE as in logreg_dense_grad_kernel.
template <bool FUSE>
__global__ __launch_bounds__(kBlock) void logreg_dense_parts_kernel(const float* __restrict__ parts,
                                                                    const float* __restrict__ w, float* __restrict__ g,
                                                                    uint64_t d, uint32_t S, float inv_b, float l2,
                                                                    ScaleFusion fuse) {
  __shared__ float red[16];
  const uint32_t m = blockIdx.y;
  const uint64_t col = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
  const bool active = col < d / 4;
  float amax = 0.f;
  if (active) {
    const float4* __restrict__ p = reinterpret_cast<const float4*>(parts + (uint64_t)m * S * d) + col;
    float4 acc = load_stream(p);
    for (uint32_t s = 1; s < S; ++s) {
      const float4 v = load_stream(p + (uint64_t)s * (d / 4));
      acc.x += v.x;
      acc.y += v.y;
      acc.z += v.z;
      acc.w += v.w;
    }
    const float4 wv = reinterpret_cast<const float4*>(w)[col];
    float4 o;
    o.x = __builtin_fmaf(l2, wv.x, acc.x * inv_b);
    o.y = __builtin_fmaf(l2, wv.y, acc.y * inv_b);
    o.z = __builtin_fmaf(l2, wv.z, acc.z * inv_b);
    o.w = __builtin_fmaf(l2, wv.w, acc.w * inv_b);
    reinterpret_cast<float4*>(g + (uint64_t)m * d)[col] = o;
    if (FUSE) {
      float4 r1, r2;
      load_refs4(fuse, col, r1, r2);
      amax = absmax4(fuse, o, r1, r2);
    }
  }
  if (FUSE) {
    amax = block_max(amax, red);
    if (threadIdx.x == 0) fuse.partials[(uint64_t)blockIdx.x * gridDim.y + m] = amax;
  }
}

// ------------------------------------------------------------------------------------------
// CSR logistic regression, column-tiled.
//
// Gathering w[col] and scattering into g[col] one stored entry at a time costs a 64-byte memory
// transaction per 4 useful bytes (measured: 9.5 ms + 26 ms per step at d = 2^24, M = 64, B = 512).
// Instead the columns are cut into tiles of 2^kCsrTileShift coordinates and a workgroup owns one
// (worker, tile): the tile of w, then the tile of g, lives in LDS, and every minibatch row
// contributes the contiguous segment of its (ascending) columns that falls into the tile.
//   1. csr_bounds_kernel   one coalesced pass over the minibatch rows' column ids: for every row
//                          and tile, the offset of the first entry at or beyond the tile start;
//   2. csr_z_kernel        per (row, tile) partial dot product sum val * w_tile[col];
//      csr_z_reduce_kernel z_i = sum of the partials over the tiles;
//   3. csr_grad_kernel     r_i = sigma(z_i) - y_i; g_tile[col] += (r_i / B) val in LDS, then the whole
//                          tile is written once (+ l2 w): no zero fill, no global atomics.
// The g tile is accumulated in fp64: on this hardware an fp32 LDS atomic add serialises over the
// lanes (~170 clocks per wavefront instruction) while the fp64 one runs at ~12; as a side effect g
// is the correctly rounded sum almost always, whatever the order of the additions.
// Entries are read twice in segment-sized pieces, g is written once.
// ------------------------------------------------------------------------------------------
constexpr int kCsrThreads = 1024;  // 16 wavefronts
constexpr int kCsrRows = 512;      // minibatch rows staged in LDS per trip
constexpr int kCsrLanes = 32;      // lanes that share one row segment (mean segment: 16 entries at 0.1 % density)
constexpr int kCsrUnroll = 16;     // row segments in flight per lane group
constexpr uint32_t kCsrGroups = kCsrThreads / kCsrLanes;
static_assert(kCsrGroups * kCsrUnroll == kCsrRows, "one sweep of the lane groups covers one trip");

// The stored entries of one worker's shard, in either of the two layouts the library takes: separate
// column and value arrays, or one array of (column, value) pairs.  With pairs a row segment of a
// tile is one contiguous piece of 8 bytes per entry instead of two pieces of 4: segments are short
// (16 entries per row and tile at 0.1 % density), and what such reads deliver is set by the 128-byte
// memory lines they touch, so one piece of twice the length moves the same entries in about two
// thirds of the line traffic, with half the load instructions.
typedef int v2i_t __attribute__((ext_vector_type(2)));
// Which column tile (of n, one per workgroup along x) workgroup bx takes.  Workgroups are handed to the
// eight compute dies in turn (bx mod 8), each die with an L2 of its own: die k gets the k-th eighth of the
// tiles, in order, so that the workgroups running side by side on a die are on ADJACENT tiles and the memory
// lines shared by the end of one tile's row segment and the start of the next tile's are fetched from HBM
// once (a bijection for any n; only the traffic depends on how the hardware really deals workgroups out).
__device__ __forceinline__ uint32_t tile_of_workgroup(uint32_t bx, uint32_t n) {
  constexpr uint32_t kDies = 8;
  if (n % kDies != 0) return bx;  // rows of the grid would start on different dies: keep the plain order
  return (bx % kDies) * (n / kDies) + bx / kDies;
}

template <bool PAIRS>
struct CsrEntries {
  GlobalPtr<int32_t> c;  // column ids, or the pairs viewed as 32-bit words (column at 2 pos, value at 2 pos + 1)
  GlobalPtr<float> v;    // values (unused with pairs)
  __device__ __forceinline__ CsrEntries(const int32_t* cols, const float* vals) : c(as_global(cols)), v(as_global(vals)) {}
  __device__ __forceinline__ int32_t col(int64_t pos) const { return PAIRS ? c[2 * pos] : c[pos]; }
  __device__ __forceinline__ void load(int64_t pos, int32_t& col, float& val) const {
    if (PAIRS) {
      const v2i_t p = reinterpret_cast<GlobalPtr<v2i_t>>(c)[pos];
      col = p.x;
      val = __int_as_float(p.y);
    } else {
      col = c[pos];
      val = v[pos];
    }
  }
  // The same without a branch: entry pos if on, else whatever lies at dummy (any 8 valid bytes, 8-byte aligned).
  __device__ __forceinline__ void load_or(bool on, int64_t pos, const void* dummy, int32_t& col, float& val) const {
    if (PAIRS) {
      const GlobalPtr<v2i_t> at = on ? reinterpret_cast<GlobalPtr<v2i_t>>(c) + pos : (GlobalPtr<v2i_t>)dummy;
      const v2i_t p = *at;
      col = p.x;
      val = __int_as_float(p.y);
    } else {
      const GlobalPtr<int32_t> ac = on ? c + pos : (GlobalPtr<int32_t>)dummy;
      const GlobalPtr<float> av = on ? v + pos : (GlobalPtr<float>)dummy;
      col = *ac;
      val = *av;
    }
  }
};

// rowbase[m][i] = position of minibatch row i in worker m's col / val arrays; bounds[m][t][i]
// (tile-major, so that a workgroup reads the bounds of all its rows contiguously) = offset within
// the row of the first entry whose column is at or beyond the start of tile t; t = 0 .. ntiles.
template <bool PAIRS>
__global__ __launch_bounds__(kBlock) void csr_bounds_kernel(const int64_t* const* __restrict__ rowptrs,
                                                            const int32_t* const* __restrict__ cols,
                                                            const uint32_t* __restrict__ idx,
                                                            int64_t* __restrict__ rowbase,
                                                            uint32_t* __restrict__ bounds, uint32_t batch,
                                                            uint32_t ntiles, uint32_t tile_shift) {
  const uint32_t m = blockIdx.y, i = blockIdx.x;
  const uint32_t row = idx[(uint64_t)m * batch + i];
  const int64_t a = as_global(rowptrs[m])[row];
  const uint32_t nnz = (uint32_t)(as_global(rowptrs[m])[row + 1] - a);
  const CsrEntries<PAIRS> e(cols[m], nullptr);
  if (threadIdx.x == 0) rowbase[(uint64_t)m * batch + i] = a;
  uint32_t* __restrict__ out = bounds + (uint64_t)m * (ntiles + 1) * batch + i;
  // entry k opens every tile after the tile of entry k-1 up to its own tile
  for (uint32_t k = threadIdx.x; k <= nnz; k += kBlock) {
    const uint32_t prev = k == 0 ? 0u : ((uint32_t)e.col(a + k - 1) >> tile_shift) + 1u;
    const uint32_t cur = k == nnz ? ntiles : ((uint32_t)e.col(a + k) >> tile_shift);
    for (uint32_t t = prev; t <= cur; ++t) out[(uint64_t)t * batch] = k;
  }
}

// One-off: the same offsets for every row of every shard, row-major (index[m][row][t]).
template <bool PAIRS>
__global__ __launch_bounds__(kBlock) void csr_tile_index_kernel(const int64_t* const* __restrict__ rowptrs,
                                                                const int32_t* const* __restrict__ cols,
                                                                const uint64_t* __restrict__ n_rows,
                                                                const uint32_t* const* __restrict__ index,
                                                                uint32_t ntiles, uint32_t tile_shift) {
  const uint32_t m = blockIdx.y;
  const uint64_t row = blockIdx.x;
  if (row >= n_rows[m]) return;
  const int64_t a = as_global(rowptrs[m])[row];
  const uint32_t nnz = (uint32_t)(as_global(rowptrs[m])[row + 1] - a);
  const CsrEntries<PAIRS> e(cols[m], nullptr);
  uint32_t* __restrict__ out = const_cast<uint32_t*>(index[m]) + row * (ntiles + 1);
  for (uint32_t k = threadIdx.x; k <= nnz; k += kBlock) {
    const uint32_t prev = k == 0 ? 0u : ((uint32_t)e.col(a + k - 1) >> tile_shift) + 1u;
    const uint32_t cur = k == nnz ? ntiles : ((uint32_t)e.col(a + k) >> tile_shift);
    for (uint32_t t = prev; t <= cur; ++t) out[t] = k;
  }
}

// Checks of caller-supplied CSR shards (tng_validate_csr).  Stage 1: the row pointers of worker m are
// non-negative, non-decreasing, end within the nnz[m] stored entries, and no row holds 2^32 entries or
// more.  Stage 2 (only launched when stage 1 found nothing, so every access below is in range): the
// column ids of every row lie in [0, d) and ascend strictly.  A violation sets a bit of *flag.
__global__ __launch_bounds__(kBlock) void csr_validate_rowptr_kernel(const int64_t* const* __restrict__ rowptrs,
                                                                     const uint64_t* __restrict__ n_rows,
                                                                     const uint64_t* __restrict__ nnz,
                                                                     uint32_t* __restrict__ flag) {
  const uint32_t m = blockIdx.y;
  const uint64_t n = n_rows[m];
  const GlobalPtr<int64_t> rp = as_global(rowptrs[m]);
  const uint64_t stride = (uint64_t)gridDim.x * kBlock;
  uint32_t bad = 0;
  for (uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += stride) {
    const int64_t a = rp[i], b = rp[i + 1];
    if (a < 0 || b < a || (uint64_t)b > nnz[m] || (uint64_t)(b - a) >= (1ull << 32)) bad = 1u;
  }
  if (bad != 0) atomicOr(flag, 1u);
}

template <bool PAIRS>
__global__ __launch_bounds__(kBlock) void csr_validate_cols_kernel(const int64_t* const* __restrict__ rowptrs,
                                                                   const int32_t* const* __restrict__ cols,
                                                                   const uint64_t* __restrict__ n_rows, uint64_t d,
                                                                   uint32_t* __restrict__ flag) {
  const uint32_t m = blockIdx.y;
  const uint64_t n = n_rows[m];
  uint32_t bad = 0;
  for (uint64_t row = blockIdx.x; row < n; row += gridDim.x) {
    const int64_t a = as_global(rowptrs[m])[row], b = as_global(rowptrs[m])[row + 1];
    const CsrEntries<PAIRS> e(cols[m], nullptr);
    for (int64_t k = a + threadIdx.x; k < b; k += kBlock) {
      const int32_t cur = e.col(k);
      if (cur < 0 || (uint64_t)cur >= d) bad |= 2u;
      if (k > a && e.col(k - 1) >= cur) bad |= 4u;
    }
  }
  if (bad != 0) atomicOr(flag, bad);
}

// Per iteration, with the index: the index rows of the minibatch are transposed into the tile-major
// bounds array (64 x 64 blocks through LDS, both sides coalesced), and rowbase is filled.
constexpr int kGatherTile = 64;
__global__ __launch_bounds__(kBlock) void csr_gather_bounds_kernel(const int64_t* const* __restrict__ rowptrs,
                                                                   const uint32_t* const* __restrict__ index,
                                                                   const uint32_t* __restrict__ idx,
                                                                   int64_t* __restrict__ rowbase,
                                                                   uint32_t* __restrict__ bounds, uint32_t batch,
                                                                   uint32_t ntiles) {
  __shared__ uint32_t tile[kGatherTile][kGatherTile + 1];
  const uint32_t m = blockIdx.z;
  const uint32_t t0 = blockIdx.x * kGatherTile, i0 = blockIdx.y * kGatherTile;
  const uint32_t tx = threadIdx.x % kGatherTile, ty = threadIdx.x / kGatherTile;
  const GlobalPtr<uint32_t> src = as_global(index[m]);
  for (uint32_t r = ty; r < (uint32_t)kGatherTile; r += kBlock / kGatherTile) {
    const uint32_t i = i0 + r;
    if (i < batch && t0 + tx <= ntiles) {
      const uint64_t row = idx[(uint64_t)m * batch + i];
      tile[r][tx] = src[row * (ntiles + 1) + t0 + tx];
    }
  }
  __syncthreads();
  for (uint32_t r = ty; r < (uint32_t)kGatherTile; r += kBlock / kGatherTile) {
    const uint32_t t = t0 + r;
    if (t <= ntiles && i0 + tx < batch) bounds[((uint64_t)m * (ntiles + 1) + t) * batch + i0 + tx] = tile[tx][r];
  }
  if (blockIdx.x == 0 && ty == 0 && i0 + tx < batch) {
    const uint64_t o = (uint64_t)m * batch + i0 + tx;
    rowbase[o] = as_global(rowptrs[m])[idx[o]];
  }
}

// Stages, for minibatch rows first .. first+count-1 of worker m, the entry range of the row that
// falls into tile t (absolute positions).
__device__ __forceinline__ void csr_stage_segments(const int64_t* __restrict__ rowbase,
                                                   const uint32_t* __restrict__ bounds, uint32_t m, uint32_t batch,
                                                   uint32_t ntiles, uint32_t t, uint32_t first, uint32_t count,
                                                   int64_t* sLo, uint32_t* sLen) {
  const uint32_t* __restrict__ b = bounds + ((uint64_t)m * (ntiles + 1) + t) * batch + first;
  const int64_t* __restrict__ base = rowbase + (uint64_t)m * batch + first;
  for (uint32_t j = threadIdx.x; j < count; j += kCsrThreads) {
    const uint32_t lo = b[j], hi = b[batch + j];
    sLo[j] = base[j] + lo;
    sLen[j] = hi - lo;
  }
}

// The first lane-width of entries of kCsrUnroll row segments, all loads issued before any is used.
struct CsrBatch {
  uint32_t len[kCsrUnroll];
  int32_t col[kCsrUnroll];
  float val[kCsrUnroll];
};

template <bool PAIRS>
__device__ __forceinline__ void csr_load_batch(const CsrEntries<PAIRS>& e, const int64_t* sLo, const uint32_t* sLen,
                                               uint32_t j0, uint32_t count, uint32_t gl, CsrBatch& b) {
#pragma unroll
  for (int u = 0; u < kCsrUnroll; ++u) {
    const uint32_t j = j0 + u;
    b.len[u] = j < count ? sLen[j] : 0u;
    b.col[u] = 0;
    b.val[u] = 0.f;
    if (gl < b.len[u]) e.load(sLo[j] + gl, b.col[u], b.val[u]);
  }
}

template <bool PAIRS>
__global__ __launch_bounds__(kCsrThreads) void csr_z_kernel(const int32_t* const* __restrict__ cols,
                                                            const float* const* __restrict__ vals,
                                                            const int64_t* __restrict__ rowbase,
                                                            const uint32_t* __restrict__ bounds,
                                                            const float* __restrict__ w, float* __restrict__ zparts,
                                                            uint64_t d, uint32_t batch, uint32_t ntiles,
                                                            uint32_t tile_shift) {
  extern __shared__ float wtile[];  // w over the tile's columns
  __shared__ __align__(16) int64_t sLo[kCsrRows];
  __shared__ __align__(16) uint32_t sLen[kCsrRows];
  // workers vary fastest across the grid: the workgroups that run side by side share one tile of w
  const uint32_t m = blockIdx.x, t = blockIdx.y;
  const uint32_t T = 1u << tile_shift;
  const uint64_t c0 = (uint64_t)t << tile_shift;
  float* __restrict__ zpart = zparts + ((uint64_t)m * ntiles + t) * batch;
  if (tile_shift == kCsrTileShift && c0 + T <= d && (reinterpret_cast<uintptr_t>(w) & 15u) == 0) {
    // full-size tile: all its loads in flight at once, then the LDS stores
    constexpr int kVec = (1 << kCsrTileShift) / (4 * kCsrThreads);
    const float4* __restrict__ w4 = reinterpret_cast<const float4*>(w + c0);
    float4* tile4 = reinterpret_cast<float4*>(wtile);
    float4 tmp[kVec];
#pragma unroll
    for (int q = 0; q < kVec; ++q) tmp[q] = w4[q * kCsrThreads + threadIdx.x];
#pragma unroll
    for (int q = 0; q < kVec; ++q) tile4[q * kCsrThreads + threadIdx.x] = tmp[q];
  } else {
    for (uint32_t j = threadIdx.x; j < T; j += kCsrThreads) wtile[j] = c0 + j < d ? w[c0 + j] : 0.f;
  }
  const CsrEntries<PAIRS> e(cols[m], vals[m]);
  const uint32_t group = threadIdx.x / kCsrLanes, gl = threadIdx.x % kCsrLanes;
  for (uint32_t first = 0; first < batch; first += kCsrRows) {
    const uint32_t count = min((uint32_t)kCsrRows, batch - first);
    __syncthreads();
    csr_stage_segments(rowbase, bounds, m, batch, ntiles, t, first, count, sLo, sLen);
    __syncthreads();
    const uint32_t j0 = group * kCsrUnroll;
    CsrBatch b;
    csr_load_batch(e, sLo, sLen, j0, count, gl, b);
    float acc[kCsrUnroll];
#pragma unroll
    for (int u = 0; u < kCsrUnroll; ++u) {
      acc[u] = gl < b.len[u] ? b.val[u] * wtile[(uint32_t)b.col[u] - (uint32_t)c0] : 0.f;
      for (uint32_t k = gl + kCsrLanes; k < b.len[u]; k += kCsrLanes) {  // rare: segments longer than the lane group
        int32_t ck;
        float vk;
        e.load(sLo[j0 + u] + k, ck, vk);
        acc[u] = __builtin_fmaf(vk, wtile[(uint32_t)ck - (uint32_t)c0], acc[u]);
      }
    }
    // 16 sums over 32 lanes by halving: after the four exchange steps lane l holds the partial sum
    // of segment (bit4 bit3 bit2 bit1 of l) over the lanes that share those bits.
    static_assert(kCsrUnroll == 16 && kCsrLanes == 32, "the exchange pattern below is for 16 sums over 32 lanes");
    float r8[8], r4[4], r2[2];
    const bool b4 = (gl & 16) != 0, b3 = (gl & 8) != 0, b2 = (gl & 4) != 0, b1 = (gl & 2) != 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) r8[k] = (b4 ? acc[k + 8] : acc[k]) + __shfl_xor(b4 ? acc[k] : acc[k + 8], 16, kWave);
#pragma unroll
    for (int k = 0; k < 4; ++k) r4[k] = (b3 ? r8[k + 4] : r8[k]) + __shfl_xor(b3 ? r8[k] : r8[k + 4], 8, kWave);
#pragma unroll
    for (int k = 0; k < 2; ++k) r2[k] = (b2 ? r4[k + 2] : r4[k]) + __shfl_xor(b2 ? r4[k] : r4[k + 2], 4, kWave);
    float r1 = (b1 ? r2[1] : r2[0]) + __shfl_xor(b1 ? r2[0] : r2[1], 2, kWave);
    r1 += __shfl_xor(r1, 1, kWave);
    const uint32_t u = (b4 ? 8u : 0u) + (b3 ? 4u : 0u) + (b2 ? 2u : 0u) + (b1 ? 1u : 0u);
    if ((gl & 1u) == 0u && j0 + u < count) zpart[first + j0 + u] = r1;
  }
}

// The same pass with two adjacent tiles of w (2^15 columns, 128 KiB) in LDS and two loads per lane and
// row: the row segments are twice as long, so fewer of the 128-byte memory lines they touch are
// partial ones.  (Random contiguous segments deliver 2.2 TB/s of useful bytes at 64 bytes per
// segment and 3.2 TB/s at 128; this pass is bound by exactly that.)  One partial sum per row and pair
// of tiles: zparts[m][pair][i].
template <bool PAIRS>
__global__ __launch_bounds__(kCsrThreads) void csr_z_wide_kernel(const int32_t* const* __restrict__ cols,
                                                                 const float* const* __restrict__ vals,
                                                                 const int64_t* __restrict__ rowbase,
                                                                 const uint32_t* __restrict__ bounds,
                                                                 const float* __restrict__ w,
                                                                 float* __restrict__ zparts, uint64_t d,
                                                                 uint32_t batch, uint32_t ntiles, uint32_t npairs,
                                                                 uint32_t M, uint32_t workers_per_block) {
  extern __shared__ float wtile[];  // w over the columns of both tiles
  __shared__ __align__(16) int64_t sLoBuf[2][kCsrRows];  // segment starts and lengths, this step's and the next one's
  __shared__ __align__(16) uint32_t sLenBuf[2][kCsrRows];
  const uint32_t pair = tile_of_workgroup(blockIdx.x, npairs);
  const uint32_t t_lo = 2 * pair, t_hi = min(2 * pair + 2, ntiles);
  constexpr uint32_t T = 2u << kCsrTileShift;
  const uint64_t c0 = (uint64_t)t_lo << kCsrTileShift;
  if (c0 + T <= d && (reinterpret_cast<uintptr_t>(w) & 15u) == 0) {
    constexpr int kVec = (int)(T / (4 * kCsrThreads));  // 8 float4 per thread, four in flight at a time
    const float4* __restrict__ w4 = reinterpret_cast<const float4*>(w + c0);
    float4* tile4 = reinterpret_cast<float4*>(wtile);
#pragma unroll
    for (int q0 = 0; q0 < kVec; q0 += 4) {
      float4 tmp[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) tmp[q] = w4[(q0 + q) * kCsrThreads + threadIdx.x];
#pragma unroll
      for (int q = 0; q < 4; ++q) tile4[(q0 + q) * kCsrThreads + threadIdx.x] = tmp[q];
    }
  } else {
    for (uint32_t j = threadIdx.x; j < T; j += kCsrThreads) wtile[j] = c0 + j < d ? w[c0 + j] : 0.f;
  }
  const uint32_t group = threadIdx.x / kCsrLanes, gl = threadIdx.x % kCsrLanes;
  const uint32_t j0 = group * kCsrUnroll;
  // The tiles of w serve several workers in turn.  A step is one trip of kCsrRows minibatch rows of one
  // worker; the segment bounds of the next step are fetched while this step's entries are on their
  // way (every thread fetches, the row index clamped, so that no load sits under a condition).
  static_assert(kCsrThreads >= kCsrRows, "one thread per staged row");
  const uint32_t m_first = blockIdx.y * workers_per_block, m_last = min(m_first + workers_per_block, M);
  const uint32_t trips = (batch + kCsrRows - 1) / kCsrRows;
  const uint32_t steps = (m_last - m_first) * trips;
  auto fetch_bounds = [&](uint32_t step, int64_t& start, uint32_t& length) {
    const uint32_t m = m_first + step / trips, first = (step % trips) * kCsrRows;
    const uint32_t j = first + min(threadIdx.x, min((uint32_t)kCsrRows, batch - first) - 1u);
    const uint32_t* __restrict__ b = bounds + (uint64_t)m * (ntiles + 1) * batch;
    const uint32_t lo = b[(uint64_t)t_lo * batch + j], hi = b[(uint64_t)t_hi * batch + j];
    start = rowbase[(uint64_t)m * batch + j] + lo;
    length = hi - lo;
  };
  int64_t next_start;
  uint32_t next_len;
  fetch_bounds(0, next_start, next_len);
  if (threadIdx.x < (uint32_t)kCsrRows) {
    sLoBuf[0][threadIdx.x] = next_start;
    sLenBuf[0][threadIdx.x] = next_len;
  }
  for (uint32_t step = 0; step < steps; ++step) {
  {
    const uint32_t m = m_first + step / trips, first = (step % trips) * kCsrRows;
    float* __restrict__ zpart = zparts + ((uint64_t)m * npairs + pair) * batch;
    const CsrEntries<PAIRS> e(cols[m], vals[m]);
    const uint32_t count = min((uint32_t)kCsrRows, batch - first);
    const int64_t* sLo = sLoBuf[step & 1];
    const uint32_t* sLen = sLenBuf[step & 1];
    __syncthreads();  // this step's bounds are in place, the other buffer is free
    fetch_bounds(min(step + 1, steps - 1), next_start, next_len);
    uint32_t len[kCsrUnroll];
    int32_t col[kCsrUnroll][2];
    float val[kCsrUnroll][2];
#pragma unroll
    for (int u = 0; u < kCsrUnroll; ++u) {  // all loads are issued before any is used
      const uint32_t j = j0 + u;
      len[u] = j < count ? sLen[j] : 0u;
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        col[u][q] = 0;
        val[u][q] = 0.f;
        if (gl + (uint32_t)q * kCsrLanes < len[u]) e.load(sLo[j] + gl + q * kCsrLanes, col[u][q], val[u][q]);
      }
    }
    float acc[kCsrUnroll];
#pragma unroll
    for (int u = 0; u < kCsrUnroll; ++u) {
      acc[u] = gl < len[u] ? val[u][0] * wtile[(uint32_t)col[u][0] - (uint32_t)c0] : 0.f;
      if (gl + kCsrLanes < len[u]) acc[u] = __builtin_fmaf(val[u][1], wtile[(uint32_t)col[u][1] - (uint32_t)c0], acc[u]);
    }
#pragma unroll
    for (int u = 0; u < kCsrUnroll; ++u) {
      if (len[u] > 2u * kCsrLanes) {  // rare: longer than what the registers hold
        const int64_t lo = sLo[j0 + u];
        for (uint32_t k = gl + 2 * kCsrLanes; k < len[u]; k += kCsrLanes) {
          int32_t ck;
          float vk;
          e.load(lo + k, ck, vk);
          acc[u] = __builtin_fmaf(vk, wtile[(uint32_t)ck - (uint32_t)c0], acc[u]);
        }
      }
    }
    float r8[8], r4[4], r2[2];
    const bool b4 = (gl & 16) != 0, b3 = (gl & 8) != 0, b2 = (gl & 4) != 0, b1 = (gl & 2) != 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) r8[k] = (b4 ? acc[k + 8] : acc[k]) + __shfl_xor(b4 ? acc[k] : acc[k + 8], 16, kWave);
#pragma unroll
    for (int k = 0; k < 4; ++k) r4[k] = (b3 ? r8[k + 4] : r8[k]) + __shfl_xor(b3 ? r8[k] : r8[k + 4], 8, kWave);
#pragma unroll
    for (int k = 0; k < 2; ++k) r2[k] = (b2 ? r4[k + 2] : r4[k]) + __shfl_xor(b2 ? r4[k] : r4[k + 2], 4, kWave);
    float r1 = (b1 ? r2[1] : r2[0]) + __shfl_xor(b1 ? r2[0] : r2[1], 2, kWave);
    r1 += __shfl_xor(r1, 1, kWave);
    const uint32_t u = (b4 ? 8u : 0u) + (b3 ? 4u : 0u) + (b2 ? 2u : 0u) + (b1 ? 1u : 0u);
    if ((gl & 1u) == 0u && j0 + u < count) zpart[first + j0 + u] = r1;
    if (threadIdx.x < (uint32_t)kCsrRows) {
      sLoBuf[(step + 1) & 1][threadIdx.x] = next_start;
      sLenBuf[(step + 1) & 1][threadIdx.x] = next_len;
    }
  }
  }
}

// r[m][i] = (sigma(z_i) - y_i) / B with z_i = sum over the tiles of the partial dot products
// zpart[m][t][i]: what the gradient pass multiplies every stored entry of row i by.  A workgroup takes
// kReduceRows rows of one worker; four groups of threads add a quarter of the partial sums each (four
// accumulators per thread, fixed order), and the quarters are added in order.
constexpr int kReduceRows = kBlock / 4;
__global__ __launch_bounds__(kBlock) void csr_z_reduce_kernel(const float* __restrict__ zpart,
                                                              const float* const* __restrict__ ys,
                                                              const uint32_t* __restrict__ idx, float* __restrict__ r,
                                                              uint32_t batch, uint32_t ntiles, float inv_b) {
  __shared__ float quarter_sum[3][kReduceRows];
  const uint32_t m = blockIdx.y;
  const uint32_t lane_row = threadIdx.x % kReduceRows, quarter = threadIdx.x / kReduceRows;
  const uint32_t i = min(blockIdx.x * kReduceRows + lane_row, batch - 1);  // clamped: every thread meets the barrier
  const uint32_t per = (ntiles + 3) / 4;
  const uint32_t t_begin = min(quarter * per, ntiles), t_end = min(t_begin + per, ntiles);
  const float* __restrict__ p = zpart + (uint64_t)m * ntiles * batch + i;
  float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
  uint32_t t = t_begin;
  for (; t + 4 <= t_end; t += 4) {
    a0 += p[(uint64_t)t * batch];
    a1 += p[(uint64_t)(t + 1) * batch];
    a2 += p[(uint64_t)(t + 2) * batch];
    a3 += p[(uint64_t)(t + 3) * batch];
  }
  for (; t < t_end; ++t) a0 += p[(uint64_t)t * batch];
  const float part = (a0 + a1) + (a2 + a3);
  if (quarter > 0) quarter_sum[quarter - 1][lane_row] = part;
  __syncthreads();
  if (quarter == 0 && blockIdx.x * kReduceRows + lane_row < batch) {
    const float z = ((part + quarter_sum[0][lane_row]) + quarter_sum[1][lane_row]) + quarter_sum[2][lane_row];
    const uint64_t o = (uint64_t)m * batch + i;
    r[o] = logistic_residual(z, as_global(ys[m])[idx[o]]) * inv_b;
  }
}

// Gradient pass: one workgroup per (worker, tile); every minibatch row adds (r_i / B) val into the
// fp64 tile in LDS, and the finished tile is written once (+ l2 w).  FUSE: the write-out also leaves
// the tile's largest |normalize(g)| for the scale pass (partials[tile][worker]), which then need not
// read g again: +0.35 ms here against a 0.7 ms pass saved at d = 2^24, M = 64.
// Where the time goes at d = 2^24, M = 64, B = 512 (2.47 ms): without the adds 2.32 ms, without the
// write-out of g 1.96 ms -- the rest is reading the entries in 66-byte segments, at the rate such
// segments are delivered at all (see the paired dot-product pass).
// Taken apart the same way, zeroing + write-out alone take 0.85 ms and staging + entry loads alone
// 1.50 ms: per compute unit the phases simply add up.  Variants that measured slower or no faster:
// prefetching the next tile's entries during the write-out (software pipelining over a run of
// tiles); tiles of half the width with two workgroups per compute unit, so that one writes while
// the other reads (2.79 ms: the segments of 33 bytes cost more than the overlap gains); fetching the
// entries of two adjacent tiles at once into registers (one wavefront per row, segment descriptors
// as wavefront-uniform values, no spills) and working through the tiles in two phases with the first
// tile's stores left in flight (2.66 ms: its loads alone 1.26 ms, its write-out alone 1.06 ms, both
// together more than their sum -- the random reads and the streaming writes compete in memory);
// a run of four tiles per workgroup with the next tile's segment bounds prefetched, the tile cleared
// by its own write-out and barriers that wait for LDS traffic only (+0.3 ms).  What the variants that
// keep a workgroup alive across tiles have in common: loads and stores share one in-order counter,
// so the wait for the next tile's entries is also a wait for the previous tile's stores to be
// acknowledged, while a workgroup that ends after its write-out leaves them to drain behind it.
template <bool FUSE, bool PAIRS>
__global__ __launch_bounds__(kCsrThreads) void csr_grad_kernel(const int32_t* const* __restrict__ cols,
                                                               const float* const* __restrict__ vals,
                                                               const int64_t* __restrict__ rowbase,
                                                               const uint32_t* __restrict__ bounds,
                                                               const float* __restrict__ resid,
                                                               const float* __restrict__ w, float* __restrict__ g,
                                                               uint64_t d, uint32_t batch, uint32_t ntiles,
                                                               uint32_t tile_shift, float l2, ScaleFusion fuse) {
  extern __shared__ double gtile[];  // g over the tile's columns, accumulated in fp64
  __shared__ __align__(16) int64_t sLo[kCsrRows];
  __shared__ __align__(16) uint32_t sLen[kCsrRows];
  __shared__ float sR[kCsrRows];
  __shared__ float red[kCsrThreads / kWave];
  const uint32_t m = blockIdx.x, t = blockIdx.y;
  const uint32_t T = 1u << tile_shift;
  const uint64_t c0 = (uint64_t)t << tile_shift;
  for (uint32_t j = threadIdx.x; j < T; j += kCsrThreads) gtile[j] = 0.0;
  // fused scale pass: the reference of the thread's columns, fetched first so that nothing waits for it
  constexpr int kPer = (1 << kCsrTileShift) / (4 * kCsrThreads);
  float4 r1[kPer], r2[kPer];
  if (FUSE) {
#pragma unroll
    for (int k = 0; k < kPer; ++k) load_refs4(fuse, c0 / 4 + (uint32_t)k * kCsrThreads + threadIdx.x, r1[k], r2[k]);
  }
  const CsrEntries<PAIRS> e(cols[m], vals[m]);
  const uint32_t group = threadIdx.x / kCsrLanes, gl = threadIdx.x % kCsrLanes;
  for (uint32_t first = 0; first < batch; first += kCsrRows) {
    const uint32_t count = min((uint32_t)kCsrRows, batch - first);
    __syncthreads();
    csr_stage_segments(rowbase, bounds, m, batch, ntiles, t, first, count, sLo, sLen);
    for (uint32_t j = threadIdx.x; j < count; j += kCsrThreads) sR[j] = resid[(uint64_t)m * batch + first + j];
    __syncthreads();
    const uint32_t j0 = group * kCsrUnroll;
    CsrBatch b;
    csr_load_batch(e, sLo, sLen, j0, count, gl, b);
    // LDS operations complete in order, so a read issued after an atomic add waits for it: the
    // residuals are read before the first add and the adds go out back to back.
    float r[kCsrUnroll];
#pragma unroll
    for (int u = 0; u < kCsrUnroll; ++u) r[u] = b.len[u] != 0 ? sR[j0 + u] : 0.f;
#pragma unroll
    for (int u = 0; u < kCsrUnroll; ++u)
      if (gl < b.len[u]) atomicAdd(&gtile[(uint32_t)b.col[u] - (uint32_t)c0], (double)(r[u] * b.val[u]));
#pragma unroll
    for (int u = 0; u < kCsrUnroll; ++u) {
      if (b.len[u] > (uint32_t)kCsrLanes) {  // rare: segments longer than the lane group
        const int64_t lo = sLo[j0 + u];
        for (uint32_t k = gl + kCsrLanes; k < b.len[u]; k += kCsrLanes) {
          int32_t ck;
          float vk;
          e.load(lo + k, ck, vk);
          atomicAdd(&gtile[(uint32_t)ck - (uint32_t)c0], (double)(r[u] * vk));
        }
      }
    }
  }
  float* __restrict__ out = g + (uint64_t)m * d;
  if (FUSE) {
    // Fused scale pass (the launcher has checked: full tiles of 2^kCsrTileShift columns, no l2 term,
    // aligned rows).  The reference of the thread's columns is fetched before the barrier, so the wait
    // for it runs while the slower wavefronts finish their adds.
    __syncthreads();
    float4* __restrict__ out4 = reinterpret_cast<float4*>(out + c0);
    float amax = 0.f;
#pragma unroll
    for (int k = 0; k < kPer; ++k) {
      const uint32_t q = (uint32_t)k * kCsrThreads + threadIdx.x;
      const float4 o = make_float4((float)gtile[4 * q], (float)gtile[4 * q + 1], (float)gtile[4 * q + 2],
                                   (float)gtile[4 * q + 3]);
      store_stream(out4 + q, o);
      amax = fmaxf(amax, absmax4(fuse, o, r1[k], r2[k]));
    }
    amax = wave_max_nonneg(amax);
    if (threadIdx.x % kWave == 0) red[threadIdx.x / kWave] = amax;
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
      for (int k = 1; k < kCsrThreads / kWave; ++k) amax = fmaxf(amax, red[k]);
      fuse.partials[(uint64_t)t * gridDim.x + m] = amax;
    }
    return;
  }
  __syncthreads();
  if (c0 + T <= d && T % 4 == 0 && l2 == 0.f && ((reinterpret_cast<uintptr_t>(out) | (d * 4)) & 15u) == 0) {
    float4* __restrict__ out4 = reinterpret_cast<float4*>(out + c0);
    for (uint32_t q = threadIdx.x; q < T / 4; q += kCsrThreads)
      store_stream(out4 + q, make_float4((float)gtile[4 * q], (float)gtile[4 * q + 1], (float)gtile[4 * q + 2],
                                         (float)gtile[4 * q + 3]));
  } else {
    for (uint32_t j = threadIdx.x; j < T; j += kCsrThreads) {
      if (c0 + j < d) out[c0 + j] = l2 != 0.f ? __builtin_fmaf(l2, w[c0 + j], (float)gtile[j]) : (float)gtile[j];
    }
  }
}

// Workgroup barrier that orders LDS traffic only: global loads and stores still in flight are not
// waited for (__syncthreads would wait until every one of them has come back).
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// The gradient pass with the fused scale pass for the common case -- full tiles, no l2 term, at most
// kCsrRows minibatch rows, 16-byte aligned rows of g -- as a software pipeline over a run of tiles of one
// worker.  With one 128 KiB workgroup per compute unit nothing else hides a tile's chain of
// dependent memory round trips (segment bounds, then entries, then the write-out), so the workgroup
// overlaps them itself:
//   while tile t's entries are added into the LDS tile, the segment bounds of tile t+1 are on their way;
//   after the barrier that ends the adds, the entries of tile t+1 are requested BEFORE tile t is written
//   out: loads and stores retire through one in-order counter, so the wait for those entries at the
//   top of the next round only has to leave the (younger) stores outstanding, and the write-out, the
//   clearing of the tile and the stores' acknowledgement all run under the entries' latency.
// The barriers order LDS traffic only.  Lanes beyond a segment's length carry an invalid column.
template <bool PAIRS, int NORM>
__global__ __launch_bounds__(kCsrThreads) void csr_grad_run_kernel(const int32_t* const* __restrict__ cols,
                                                                   const float* const* __restrict__ vals,
                                                                   const int64_t* __restrict__ rowbase,
                                                                   const uint32_t* __restrict__ bounds,
                                                                   const float* __restrict__ resid,
                                                                   float* __restrict__ g, uint64_t d, uint32_t batch,
                                                                   uint32_t ntiles, ScaleFusion fuse) {
  extern __shared__ double gtile[];  // g over the tile's columns, accumulated in fp64
  __shared__ __align__(16) int64_t sLoBuf[2][kCsrRows];
  __shared__ __align__(16) uint32_t sLenBuf[2][kCsrRows];
  __shared__ float sR[kCsrRows];
  __shared__ float red[kCsrThreads / kWave];
  constexpr uint32_t T = 1u << kCsrTileShift;
  constexpr int kPer = (int)(T / (4 * kCsrThreads));
  const uint32_t m = blockIdx.x;
  // Workgroup r of a worker takes tiles r, r + stride, r + 2 stride, ... (stride = workgroups per worker):
  // the workgroups of one worker that run side by side are then on ADJACENT tiles, and the 128-byte memory
  // lines that hold the end of one tile's row segment and the start of the next tile's are fetched from
  // HBM once and shared in the caches (with consecutive tiles per workgroup they were fetched twice, a
  // round apart: 7.8 GB read per launch instead of 4.6 at d = 2^24, 64 workers).
  const uint32_t stride = gridDim.y;
  const uint32_t t_first = blockIdx.y;
  const uint32_t row = min(threadIdx.x, batch - 1);  // every thread fetches bounds: no load under a condition
  const uint32_t* __restrict__ b = bounds + (uint64_t)m * (ntiles + 1) * batch + row;
  const int64_t base = rowbase[(uint64_t)m * batch + row];
  const bool has_row = threadIdx.x < batch;
  {
    const uint32_t lo = b[(uint64_t)t_first * batch], hi = b[(uint64_t)(t_first + 1) * batch];
    for (uint32_t j = threadIdx.x; j < T; j += kCsrThreads) gtile[j] = 0.0;
    if (threadIdx.x < (uint32_t)kCsrRows) {
      sR[threadIdx.x] = has_row ? resid[(uint64_t)m * batch + threadIdx.x] : 0.f;
      sLoBuf[0][threadIdx.x] = base + lo;
      sLenBuf[0][threadIdx.x] = has_row ? hi - lo : 0u;
    }
  }
  const CsrEntries<PAIRS> e(cols[m], vals[m]);
  const uint32_t group = threadIdx.x / kCsrLanes, gl = threadIdx.x % kCsrLanes;
  const uint32_t j0 = group * kCsrUnroll;
  float* __restrict__ out = g + (uint64_t)m * d;
  int32_t ncol[kCsrUnroll];
  float nval[kCsrUnroll];
  uint32_t nmask = 0;  // bit u: this lane holds an entry of segment u
  uint32_t nlong = 0;  // bit u: segment u is longer than the lane group
  // The first lane-width of entries of the group's segments.  Lanes beyond a segment's length read a
  // harmless valid address (the worker's first row start) instead of skipping the load: the compiler
  // cannot count loads that sit under a condition, and would then make every later wait a wait for all.
  const void* dummy = rowbase + (uint64_t)m * batch;
  auto request = [&](uint32_t buf) {
    nmask = 0;
    nlong = 0;
#pragma unroll
    for (int u = 0; u < kCsrUnroll; ++u) {
      const uint32_t len = sLenBuf[buf][j0 + u];
      const bool on = gl < len;
      e.load_or(on, sLoBuf[buf][j0 + u] + gl, dummy, ncol[u], nval[u]);
      nmask |= on ? 1u << u : 0u;
      nlong |= len > (uint32_t)kCsrLanes ? 1u << u : 0u;
    }
  };
  auto store_maximum = [&](uint32_t t) {  // by thread 0, once red holds tile t's wavefront maxima
    float mx = red[0];
#pragma unroll
    for (int k = 1; k < kCsrThreads / kWave; ++k) mx = fmaxf(mx, red[k]);
    fuse.partials[(uint64_t)t * gridDim.x + m] = mx;
  };
  auto round = [&](uint32_t t) {
    const uint32_t cur = ((t - t_first) / stride) & 1u;
    const uint64_t c0 = (uint64_t)t << kCsrTileShift;
    // bounds of the workgroup's next tile (clamped: a fetch, never a branch); past its last tile the lengths become 0
    const bool more = t + stride < ntiles;
    const uint32_t tn = more ? t + stride : t;
    const uint32_t nlo = b[(uint64_t)tn * batch], nhi = b[(uint64_t)(tn + 1) * batch];
    // LDS operations complete in order: the residuals are read before the first add
    float r[kCsrUnroll];
#pragma unroll
    for (int u = 0; u < kCsrUnroll; ++u) r[u] = sR[j0 + u];
#pragma unroll
    for (int u = 0; u < kCsrUnroll; ++u)
      if ((nmask >> u) & 1u) atomicAdd(&gtile[(uint32_t)ncol[u] - (uint32_t)c0], (double)(r[u] * nval[u]));
    if (nlong != 0) {  // rare: segments longer than the lane group
#pragma unroll
      for (int u = 0; u < kCsrUnroll; ++u) {
        if ((nlong >> u) & 1u) {
          const uint32_t len = sLenBuf[cur][j0 + u];
          const int64_t lo = sLoBuf[cur][j0 + u];
          for (uint32_t k = gl + kCsrLanes; k < len; k += kCsrLanes) {
            int32_t ck;
            float vk;
            e.load(lo + k, ck, vk);
            atomicAdd(&gtile[(uint32_t)ck - (uint32_t)c0], (double)(r[u] * vk));
          }
        }
      }
    }
    if (threadIdx.x < (uint32_t)kCsrRows) {
      sLoBuf[cur ^ 1u][threadIdx.x] = base + nlo;
      sLenBuf[cur ^ 1u][threadIdx.x] = (has_row && more) ? nhi - nlo : 0u;
    }
    lds_barrier();  // every add of tile t has been made; the segments of tile t+1 are staged
    if (t > t_first && threadIdx.x == 0) store_maximum(t - stride);  // older than the request below: need not be counted
    // the reference of the thread's columns for the fused scale pass, asked for ahead of the entries (loads
    // come back in order: asked for after them, its arrival would be theirs); the kind of normalisation is a
    // template argument so that no branch surrounds these loads either
    float4 r1[kPer], r2[kPer];
#pragma unroll
    for (int k = 0; k < kPer; ++k)
      load_refs4_t<NORM>(fuse, c0 / 4 + (uint32_t)k * kCsrThreads + threadIdx.x, r1[k], r2[k]);
    request(cur ^ 1u);  // before the stores below
    float4* __restrict__ out4 = reinterpret_cast<float4*>(out + c0);
    float amax = 0.f;
#pragma unroll
    for (int k = 0; k < kPer; ++k) {
      const uint32_t q = (uint32_t)k * kCsrThreads + threadIdx.x;
      const float4 o = make_float4((float)gtile[4 * q], (float)gtile[4 * q + 1], (float)gtile[4 * q + 2],
                                   (float)gtile[4 * q + 3]);
      gtile[4 * q] = gtile[4 * q + 1] = gtile[4 * q + 2] = gtile[4 * q + 3] = 0.0;
      store_stream(out4 + q, o);
      amax = fmaxf(amax, absmax4_t<NORM>(fuse, o, r1[k], r2[k]));
    }
    amax = wave_max_nonneg(amax);
    if (threadIdx.x % kWave == 0) red[threadIdx.x / kWave] = amax;
    lds_barrier();  // the tile is clear again; red is complete
  };
  lds_barrier();
  request(0);
  // The first round stands apart from the loop: at the loop's head the compiler takes the weaker of what
  // its two ways in allow to stay in flight, and only after a write-out are there stores that may.
  round(t_first);
  uint32_t t_last = t_first;
  for (uint32_t t = t_first + stride; t < ntiles; t += stride) {
    round(t);
    t_last = t;
  }
  if (threadIdx.x == 0) store_maximum(t_last);
}

// The same pipeline turned by ninety degrees: a workgroup stays on ONE column tile and takes the workers
// m_first .. m_end - 1 in turn.  What a round needs of its worker -- segment bounds, row starts and
// residuals of the minibatch rows, the shard's entry array -- is fetched during the round before, as the
// next tile's bounds are above; what belongs to the tile -- the reference of the thread's columns for the
// fused scale pass -- is fetched once and stays in registers, where the kernel above asks for it again
// every round (64 workers: the reference read 64 times over, a quarter more load instructions per round
// in a kernel bound by how fast a compute unit issues them; gradient pass 2.34 -> 2.13 ms at d = 2^24).
// Workgroups that run side by side are on adjacent tiles of the same worker, so the memory lines shared
// by the end of one tile's row segment and the start of the next tile's are still fetched once.
template <bool PAIRS, int NORM>
__global__ __launch_bounds__(kCsrThreads) void csr_grad_workers_kernel(const int32_t* const* __restrict__ cols,
                                                                       const float* const* __restrict__ vals,
                                                                       const int64_t* __restrict__ rowbase,
                                                                       const uint32_t* __restrict__ bounds,
                                                                       const float* __restrict__ resid,
                                                                       float* __restrict__ g, uint64_t d, uint32_t batch,
                                                                       uint32_t ntiles, uint32_t M, uint32_t per_group,
                                                                       ScaleFusion fuse) {
  extern __shared__ double gtile[];  // g over the tile's columns, accumulated in fp64
  __shared__ __align__(16) int64_t sLoBuf[2][kCsrRows];
  __shared__ __align__(16) uint32_t sLenBuf[2][kCsrRows];
  __shared__ float sRBuf[2][kCsrRows];
  __shared__ float red[2][kCsrThreads / kWave];  // by parity of the round: read in the round after it was written
  constexpr uint32_t T = 1u << kCsrTileShift;
  constexpr int kPer = (int)(T / (4 * kCsrThreads));
  const uint32_t t = tile_of_workgroup(blockIdx.x, ntiles);
  const uint32_t m_first = blockIdx.y * per_group;
  const uint32_t m_end = min(m_first + per_group, M);
  const uint64_t c0 = (uint64_t)t << kCsrTileShift;
  const uint32_t row = min(threadIdx.x, batch - 1);  // every thread fetches its row's data: no load under a condition
  const bool has_row = threadIdx.x < batch;
  // Per-worker arrays are addressed as (wavefront-uniform start of the worker's part) + (the thread's 32-bit
  // offset): no per-thread 64-bit pointer has to live across the rounds (registers are what this kernel is
  // short of, and a spilled pointer's reload at the head of a round would wait for every load in flight).
  const uint64_t per_worker = (uint64_t)(ntiles + 1) * batch;
  const uint32_t tb_row = t * batch + row;  // bounds of worker m, this tile, this row: bounds[m per_worker + tb_row]
  auto bounds_of = [&](uint32_t m) { return as_global(bounds + (uint64_t)m * per_worker); };
  auto rowbase_of = [&](uint32_t m) { return as_global(rowbase + (uint64_t)m * batch); };
  auto resid_of = [&](uint32_t m) { return as_global(resid + (uint64_t)m * batch); };
  {
    const uint32_t lo = bounds_of(m_first)[tb_row], hi = bounds_of(m_first)[tb_row + batch];
    const int64_t base = rowbase_of(m_first)[row];
    const float res = resid_of(m_first)[row];
    for (uint32_t j = threadIdx.x; j < T; j += kCsrThreads) gtile[j] = 0.0;
    if (threadIdx.x < (uint32_t)kCsrRows) {
      sRBuf[0][threadIdx.x] = has_row ? res : 0.f;
      sLoBuf[0][threadIdx.x] = base + lo;
      sLenBuf[0][threadIdx.x] = has_row ? hi - lo : 0u;
    }
  }
  // the reference of the thread's columns: the same for every worker
  float4 r1[kPer], r2[kPer];
#pragma unroll
  for (int k = 0; k < kPer; ++k)
    load_refs4_t<NORM>(fuse, c0 / 4 + (uint32_t)k * kCsrThreads + threadIdx.x, r1[k], r2[k]);
  const uint32_t group = threadIdx.x / kCsrLanes, gl = threadIdx.x % kCsrLanes;
  const uint32_t j0 = group * kCsrUnroll;
  int32_t ncol[kCsrUnroll];
  float nval[kCsrUnroll];
  uint32_t nmask = 0;  // bit u: this lane holds an entry of segment u
  uint32_t nlong = 0;  // bit u: segment u is longer than the lane group
  // entries of worker mr's segments staged in buffer buf; lanes beyond a segment read the worker's first
  // row start instead (a load, never a branch)
  auto request = [&](const CsrEntries<PAIRS>& e, uint32_t mr, uint32_t buf) {
    const void* dummy = rowbase + (uint64_t)mr * batch;
    nmask = 0;
    nlong = 0;
#pragma unroll
    for (int u = 0; u < kCsrUnroll; ++u) {
      const uint32_t len = sLenBuf[buf][j0 + u];
      const bool on = gl < len;
      e.load_or(on, sLoBuf[buf][j0 + u] + gl, dummy, ncol[u], nval[u]);
      nmask |= on ? 1u << u : 0u;
      nlong |= len > (uint32_t)kCsrLanes ? 1u << u : 0u;
    }
  };
  auto store_maximum = [&](uint32_t m) {  // by thread 0, once red holds worker m's wavefront maxima
    const float* rm = red[(m - m_first) & 1u];
    float mx = rm[0];
#pragma unroll
    for (int k = 1; k < kCsrThreads / kWave; ++k) mx = fmaxf(mx, rm[k]);
    fuse.partials[(uint64_t)t * M + m] = mx;
  };
  auto round = [&](uint32_t m) {
    const uint32_t cur = (m - m_first) & 1u;
    // what the next worker's round needs (worker index clamped: a fetch, never a branch); past the last
    // worker the lengths become 0
    const bool more = m + 1 < m_end;
    const uint32_t mn = more ? m + 1 : m;
    const uint32_t nlo = bounds_of(mn)[tb_row], nhi = bounds_of(mn)[tb_row + batch];
    const int64_t nbase = rowbase_of(mn)[row];
    const float nres = resid_of(mn)[row];
    const CsrEntries<PAIRS> e(cols[m], vals[m]), en(cols[mn], vals[mn]);
    // LDS operations complete in order: the residuals are read before the first add
    float r[kCsrUnroll];
#pragma unroll
    for (int u = 0; u < kCsrUnroll; ++u) r[u] = sRBuf[cur][j0 + u];
#pragma unroll
    for (int u = 0; u < kCsrUnroll; ++u) {
      if ((nmask >> u) & 1u) atomicAdd(&gtile[(uint32_t)ncol[u] - (uint32_t)c0], (double)(r[u] * nval[u]));
      // four adds at a time: all sixteen addresses and binary64 terms at once do not fit next to the reference
      if (u % 4 == 3) asm volatile("" ::: "memory");
    }
    if (nlong != 0) {  // rare: segments longer than the lane group
#pragma unroll
      for (int u = 0; u < kCsrUnroll; ++u) {
        if ((nlong >> u) & 1u) {
          const uint32_t len = sLenBuf[cur][j0 + u];
          const int64_t lo = sLoBuf[cur][j0 + u];
          for (uint32_t k = gl + kCsrLanes; k < len; k += kCsrLanes) {
            int32_t ck;
            float vk;
            e.load(lo + k, ck, vk);
            atomicAdd(&gtile[(uint32_t)ck - (uint32_t)c0], (double)(r[u] * vk));
          }
        }
      }
    }
    if (threadIdx.x < (uint32_t)kCsrRows) {
      sRBuf[cur ^ 1u][threadIdx.x] = has_row ? nres : 0.f;
      sLoBuf[cur ^ 1u][threadIdx.x] = nbase + nlo;
      sLenBuf[cur ^ 1u][threadIdx.x] = (has_row && more) ? nhi - nlo : 0u;
    }
    lds_barrier();  // every add of worker m has been made; the segments of worker m+1 are staged
    if (m > m_first && threadIdx.x == 0) store_maximum(m - 1);  // older than the request below: need not be counted
    request(en, mn, cur ^ 1u);  // before the stores below
    float4* __restrict__ out4 = reinterpret_cast<float4*>(g + (uint64_t)m * d + c0);
    float amax = 0.f;
#pragma unroll
    for (int k = 0; k < kPer; ++k) {
      const uint32_t q = (uint32_t)k * kCsrThreads + threadIdx.x;
      const float4 o = make_float4((float)gtile[4 * q], (float)gtile[4 * q + 1], (float)gtile[4 * q + 2],
                                   (float)gtile[4 * q + 3]);
      gtile[4 * q] = gtile[4 * q + 1] = gtile[4 * q + 2] = gtile[4 * q + 3] = 0.0;
      store_stream(out4 + q, o);
      amax = fmaxf(amax, absmax4_t<NORM>(fuse, o, r1[k], r2[k]));
    }
    amax = wave_max_nonneg(amax);
    if (threadIdx.x % kWave == 0) red[cur][threadIdx.x / kWave] = amax;
    lds_barrier();  // the tile is clear again; red is complete
  };
  lds_barrier();
  request(CsrEntries<PAIRS>(cols[m_first], vals[m_first]), m_first, 0);
  // the first round stands apart from the loop, as in the kernel above
  round(m_first);
  for (uint32_t m = m_first + 1; m < m_end; ++m) round(m);
  if (threadIdx.x == 0) store_maximum(m_end - 1);
}

// Chain Rosenbrock gradient ("Nonconvex Problems", d-dimensional form) plus per-worker noise.
// Fixed expression tree, one rounding per operation:
//   a = x[i+1] - x[i]*x[i];  t1 = (-400*x[i])*a;  t2 = -2*(1 - x[i])        (i < d-1)
//   b = x[i] - x[i-1]*x[i-1];  t3 = 200*b                                    (i > 0)
//   g = ((t1 + t2) + t3) + noise, absent terms left out.
__device__ __forceinline__ float rosenbrock_component(float xp, float xi, float xn, bool has_prev, bool has_next) {
  float base = 0.f;
  if (has_next) {
    const float a = xn - xi * xi;
    const float t1 = (-400.0f * xi) * a;
    const float t2 = -2.0f * (1.0f - xi);
    base = t1 + t2;
  }
  if (has_prev) {
    const float b = xi - xp * xp;
    const float t3 = 200.0f * b;
    base = has_next ? base + t3 : t3;
  }
  return base;
}

// Four standard normal deviates times sigma from one Philox block (Box-Muller; see NoiseGen).  The
// angle is handed to sincospi as the exact number 2 u2, so there is no argument-reduction error.
__device__ __forceinline__ float4 gaussian4(const NoiseGen& gen, uint64_t block, uint32_t m) {
  const U32x4 r = philox4x32_10((uint32_t)block, m, gen.iter, 2u, gen.k0, gen.k1);
  const float ua = (float)((r.x >> 8) + 1u) * 0x1p-24f, ub = (float)((r.z >> 8) + 1u) * 0x1p-24f;
  const float ra = sqrtf(-2.0f * logf(ua)), rb = sqrtf(-2.0f * logf(ub));
  float sa, ca, sb, cb;
  sincospif(2.0f * uniform24(r.y), &sa, &ca);
  sincospif(2.0f * uniform24(r.w), &sb, &cb);
  return make_float4(gen.sigma * (ra * ca), gen.sigma * (ra * sa), gen.sigma * (rb * cb), gen.sigma * (rb * sb));
}

__global__ __launch_bounds__(kBlock) void rosenbrock_kernel(const float* __restrict__ x,
                                                            const float* __restrict__ noise, NoiseGen gen,
                                                            float* __restrict__ g, uint64_t first, uint64_t d,
                                                            uint32_t M) {
  const uint64_t stride = (uint64_t)gridDim.x * kBlock;
  for (uint64_t i = first + (uint64_t)blockIdx.x * kBlock + threadIdx.x; i < d; i += stride) {
    const float base = rosenbrock_component(i > 0 ? x[i - 1] : 0.f, x[i], i + 1 < d ? x[i + 1] : 0.f, i > 0, i + 1 < d);
    for (uint32_t m = 0; m < M; ++m) {
      const uint64_t o = (uint64_t)m * d + i;
      if (gen.sigma > 0.f) {
        const float4 z = gaussian4(gen, i >> 2, m);
        const uint32_t c = (uint32_t)(i & 3);
        g[o] = base + (c == 0 ? z.x : c == 1 ? z.y : c == 2 ? z.z : z.w);
      } else {
        g[o] = noise != nullptr ? base + noise[o] : base;
      }
    }
  }
}

// The first 4 * (d / 4) coordinates: a thread owns 4 consecutive ones; the gradient is computed once
// and reused for all workers, the noise is streamed with 16-byte loads (rows of noise and g start at
// any 4-byte boundary when d is not a multiple of 4).
template <bool FUSE>
__global__ __launch_bounds__(kBlock) void rosenbrock_vec_kernel(const float* __restrict__ x,
                                                                const float* __restrict__ noise, NoiseGen gen,
                                                                float* __restrict__ g, uint64_t d, uint32_t M,
                                                                ScaleFusion fuse) {
  constexpr int MC = 8;  // workers per trip: their noise loads are all in flight before the first is used
  __shared__ float red[kWavesPerBlock][MC];
  const uint64_t nvec = d / 4;
  const uint64_t q = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
  const bool active = q < nvec;
  const uint64_t qc = active ? q : nvec - 1;  // idle threads of the last workgroup repeat its last float4 (and store nothing)
  float4 base, r1, r2;
  {
    const float4 xv = reinterpret_cast<const float4*>(x)[qc];
    const bool first = qc == 0, last = 4 * qc + 4 >= d;
    const float xl = first ? 0.f : x[4 * qc - 1];
    const float xr = last ? 0.f : x[4 * qc + 4];
    base.x = rosenbrock_component(xl, xv.x, xv.y, !first, true);
    base.y = rosenbrock_component(xv.x, xv.y, xv.z, true, true);
    base.z = rosenbrock_component(xv.y, xv.z, xv.w, true, true);
    base.w = rosenbrock_component(xv.z, xv.w, xr, true, !last);
    r1 = r2 = make_float4(0.f, 0.f, 0.f, 0.f);
    if (FUSE) load_refs4(fuse, qc, r1, r2);
  }
  const bool from_tensor = !(gen.sigma > 0.f) && noise != nullptr;
  const bool generated = gen.sigma > 0.f;
  for (uint32_t m0 = 0; m0 < M; m0 += MC) {
    float4 n[MC];
    if (from_tensor) {
#pragma unroll
      for (int k = 0; k < MC; ++k)  // worker index clamped: a load, never a branch
        n[k] = load4_stream_any(as_global(noise) + (uint64_t)min(m0 + k, M - 1) * d, qc);
    }
    float amax[MC];
#pragma unroll
    for (int k = 0; k < MC; ++k) {
      amax[k] = 0.f;
      if (m0 + k < M) {
        float4 o = base;
        if (generated) n[k] = gaussian4(gen, qc, m0 + k);
        if (generated || from_tensor) {
          o.x = base.x + n[k].x;
          o.y = base.y + n[k].y;
          o.z = base.z + n[k].z;
          o.w = base.w + n[k].w;
        }
        if (active) {
          store4_any(g + (uint64_t)(m0 + k) * d, q, o);
          if (FUSE) amax[k] = absmax4(fuse, o, r1, r2);
        }
      }
    }
    if (FUSE) {  // the workgroup's maxima of the trip's workers with one pair of barriers
      const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
#pragma unroll
      for (int k = 0; k < MC; ++k) {
        const float v = wave_max_nonneg(amax[k]);
        if (lane == 0) red[wave][k] = v;
      }
      __syncthreads();
      if (threadIdx.x < (uint32_t)MC && m0 + threadIdx.x < M) {
        float v = red[0][threadIdx.x];
#pragma unroll
        for (int wv = 1; wv < kWavesPerBlock; ++wv) v = fmaxf(v, red[wv][threadIdx.x]);
        fuse.partials[(uint64_t)blockIdx.x * M + m0 + threadIdx.x] = v;
      }
      __syncthreads();  // red is reused by the next trip
    }
  }
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

hipError_t launch_minibatch_indices(uint32_t k0, uint32_t k1, uint32_t iter, uint32_t M, uint32_t batch,
                                    const uint64_t* n_rows, uint32_t* idx, hipStream_t s) {
  dim3 grid((batch + kBlock - 1) / kBlock, M);
  hipLaunchKernelGGL(minibatch_indices_kernel, grid, dim3(kBlock), 0, s, k0, k1, iter, batch, n_rows, idx);
  return hipGetLastError();
}

uint32_t dense_row_splits(uint64_t d, uint32_t M, uint32_t batch) {
  // one pass over whole rows kept on chip: rows of 16 K to 64 K columns (shorter ones leave the threads too
  // little to do, longer ones do not fit), 16-byte aligned, and enough rows for two or more per workgroup
  // (between 32 K and 64 K columns only the full width: the masked form of the widest variant does not fit the
  // register file)
  if (d % 4 != 0 || d < 16384 || (d > 32768 && d != 65536) || (uint64_t)M * batch < 512) return 0;
  uint32_t S = 256 / (M < 256 ? M : 256);
  S = S < 1 ? 1 : S;
  return S < batch ? S : batch;
}

hipError_t launch_logreg_dense_grad(const LogregData& p, uint64_t d, uint32_t M, uint32_t batch, float l2,
                                    uint32_t k0, uint32_t k1, uint32_t iter, uint32_t* idx, float* resid,
                                    float* parts, const float* w, float* g, const ScaleFusion* fuse,
                                    uint32_t* fused_rows, hipStream_t s) {
  if (fused_rows != nullptr) *fused_rows = 0;
  const uint32_t S = parts != nullptr && aligned16(w) && aligned16(g) ? dense_row_splits(d, M, batch) : 0;
  if (S != 0) {
    const int nv = d <= 16384 ? 8 : d <= 32768 ? 16 : 32;
    const bool full = d / 4 == (uint64_t)nv * kRowsThreads;
    const size_t lds = (size_t)(nv < kRowsLds ? nv : kRowsLds) * kRowsThreads * sizeof(float4);
    const void* fns[] = {reinterpret_cast<const void*>(logreg_dense_rows_kernel<8, false>),
                         reinterpret_cast<const void*>(logreg_dense_rows_kernel<8, true>),
                         reinterpret_cast<const void*>(logreg_dense_rows_kernel<16, false>),
                         reinterpret_cast<const void*>(logreg_dense_rows_kernel<16, true>),
                         reinterpret_cast<const void*>(logreg_dense_rows_kernel<32, true>),  // 32 float4 per thread:
                         reinterpret_cast<const void*>(logreg_dense_rows_kernel<32, true>)};  // d = 2^16 only, always full
    {  // 128 KiB of dynamic LDS: raised once per device
      static std::mutex attr_mutex;
      static bool attr_done[64] = {};
      int dev = -1;
      if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
      std::lock_guard<std::mutex> attr_lock(attr_mutex);
      if (!attr_done[dev]) {
        for (const void* fn : fns) {
          const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize,
                                                   kRowsLds * kRowsThreads * (int)sizeof(float4));
          if (e != hipSuccess) return e;
        }
        attr_done[dev] = true;
      }
    }
    const dim3 grid(S, M);
    void* args[] = {(void*)&p.X, (void*)&p.y, (void*)&p.n_rows, (void*)&idx, (void*)&w, (void*)&parts,
                    (void*)&d,   (void*)&batch, (void*)&k0, (void*)&k1, (void*)&iter};
    const int which = (nv == 8 ? 0 : nv == 16 ? 2 : 4) + (full ? 1 : 0);
    const hipError_t el = hipLaunchKernel(fns[which], grid, dim3(kRowsThreads), args, lds, s);
    if (el != hipSuccess) return el;
    const float inv_batch = 1.0f / (float)batch;
    dim3 grid_p((uint32_t)((d / 4 + kBlock - 1) / kBlock), M);
    if (fuse != nullptr && fused_rows != nullptr && grid_p.x <= kAbsmaxMaxBlocks && aligned16(fuse->gref) &&
        aligned16(fuse->gref2)) {
      hipLaunchKernelGGL(logreg_dense_parts_kernel<true>, grid_p, dim3(kBlock), 0, s, parts, w, g, d, S, inv_batch, l2, *fuse);
      *fused_rows = grid_p.x;
    } else {
      hipLaunchKernelGGL(logreg_dense_parts_kernel<false>, grid_p, dim3(kBlock), 0, s, parts, w, g, d, S, inv_batch, l2,
                         ScaleFusion{});
    }
    return hipGetLastError();
  }
  // Rows of X and of g start at any 4-byte boundary when d is not a multiple of 4: the vector kernels
  // read and write them with 16-byte accesses that assume no more, over the first 4 * (d / 4) columns.
  const bool vec = d >= 4 && aligned16(w);
  const bool whole = d % 4 == 0;
  const float inv_b = 1.0f / (float)batch;
  dim3 grid_r(batch, M);
  if (vec && (uint64_t)M * (batch / 4) >= 1024) {  // enough rows to keep the chip busy four at a time
    hipLaunchKernelGGL((logreg_dense_resid_kernel<true, 4>), dim3((batch + 3) / 4, M), dim3(kBlock), 0, s, p.X, p.y,
                       p.n_rows, idx, w, resid, d, batch, k0, k1, iter);
  } else if (vec) {
    hipLaunchKernelGGL((logreg_dense_resid_kernel<true, 1>), grid_r, dim3(kBlock), 0, s, p.X, p.y, p.n_rows, idx, w, resid,
                       d, batch, k0, k1, iter);
  }
  if (vec) {
    dim3 grid_g((uint32_t)((d / 4 + kBlock - 1) / kBlock), M);
    // the fused scale pass sees the vector part only, so it needs all of d there
    const bool can_fuse = whole && fuse != nullptr && fused_rows != nullptr && grid_g.x <= kAbsmaxMaxBlocks &&
                          aligned16(fuse->gref) && aligned16(fuse->gref2);
    if (whole && aligned16(g)) {  // a handful of workgroups: split the rows
      const uint32_t narrow = (uint32_t)((d / 4 + 31) / 32);
#define TNG_SPLIT(COLS, GX, F)                                                                                        \
  hipLaunchKernelGGL((logreg_dense_grad_split_kernel<COLS, F>), dim3(GX, M), dim3(kSplitThreads), 0, s, p.X, idx, resid, \
                     w, g, d, batch, inv_b, l2, F ? *fuse : ScaleFusion{})
      if (narrow <= 8 && batch >= 64) {  // d <= 1024; up to 8 rows of fused maxima are reduced by the quantiser itself
        if (can_fuse) {
          TNG_SPLIT(32, narrow, true);
          *fused_rows = narrow;
        } else {
          TNG_SPLIT(32, narrow, false);
        }
        return hipGetLastError();
      }
      if ((uint64_t)grid_g.x * M <= 128 && batch >= 16) {
        if (can_fuse) {
          TNG_SPLIT(256, grid_g.x, true);
          *fused_rows = grid_g.x;
        } else {
          TNG_SPLIT(256, grid_g.x, false);
        }
        return hipGetLastError();
      }
#undef TNG_SPLIT
    }
    if (can_fuse) {
      hipLaunchKernelGGL((logreg_dense_grad_kernel<true, true>), grid_g, dim3(kBlock), 0, s, p.X, idx, resid, w, g, d,
                         (uint64_t)0, batch, inv_b, l2, *fuse);
      *fused_rows = grid_g.x;
    } else {
      hipLaunchKernelGGL((logreg_dense_grad_kernel<true, false>), grid_g, dim3(kBlock), 0, s, p.X, idx, resid, w, g, d,
                         (uint64_t)0, batch, inv_b, l2, ScaleFusion{});
    }
    if (!whole)  // the last d mod 4 columns
      hipLaunchKernelGGL((logreg_dense_grad_kernel<false, false>), dim3(1, M), dim3(kBlock), 0, s, p.X, idx, resid, w, g,
                         d, 4 * (d / 4), batch, inv_b, l2, ScaleFusion{});
  } else {
    hipLaunchKernelGGL((logreg_dense_resid_kernel<false, 1>), grid_r, dim3(kBlock), 0, s, p.X, p.y, p.n_rows, idx, w,
                       resid, d, batch, k0, k1, iter);
    dim3 grid_g((uint32_t)((d + kBlock - 1) / kBlock), M);
    hipLaunchKernelGGL((logreg_dense_grad_kernel<false, false>), grid_g, dim3(kBlock), 0, s, p.X, idx, resid, w, g, d,
                       (uint64_t)0, batch, inv_b, l2, ScaleFusion{});
  }
  return hipGetLastError();
}

uint32_t csr_tile_shift(uint64_t d) {
  uint32_t shift = kCsrTileShift;
  while (shift > 8 && (1ull << (shift - 1)) >= d) --shift;  // small problems: one tile just covering d
  return shift;
}

uint32_t csr_tiles(uint64_t d) {
  const uint32_t shift = csr_tile_shift(d);
  return (uint32_t)((d + (1ull << shift) - 1) >> shift);
}

hipError_t launch_csr_validate_rowptr(const LogregData& p, uint32_t M, uint64_t max_rows, const uint64_t* nnz,
                                      uint32_t* flag, hipStream_t s) {
  const uint64_t bx = (max_rows + kBlock - 1) / kBlock;
  hipLaunchKernelGGL(csr_validate_rowptr_kernel, dim3((uint32_t)(bx < 4096 ? bx : 4096), M), dim3(kBlock), 0, s, p.rowptr,
                     p.n_rows, nnz, flag);
  return hipGetLastError();
}

hipError_t launch_csr_validate_cols(const LogregData& p, uint64_t d, uint32_t M, uint64_t max_rows, uint32_t* flag,
                                    hipStream_t s) {
  const dim3 grid((uint32_t)(max_rows < 65535 ? max_rows : 65535), M);
  if (p.pairs)
    hipLaunchKernelGGL(csr_validate_cols_kernel<true>, grid, dim3(kBlock), 0, s, p.rowptr, p.col, p.n_rows, d, flag);
  else
    hipLaunchKernelGGL(csr_validate_cols_kernel<false>, grid, dim3(kBlock), 0, s, p.rowptr, p.col, p.n_rows, d, flag);
  return hipGetLastError();
}

hipError_t launch_csr_tile_index(const LogregData& p, uint64_t d, uint32_t M, uint64_t max_rows, hipStream_t s) {
  if (max_rows == 0 || max_rows > 0x7fffffffull || p.tile_index == nullptr) return hipErrorInvalidValue;
  const dim3 grid((uint32_t)max_rows, M);
  if (p.pairs)
    hipLaunchKernelGGL(csr_tile_index_kernel<true>, grid, dim3(kBlock), 0, s, p.rowptr, p.col, p.n_rows, p.tile_index,
                       csr_tiles(d), csr_tile_shift(d));
  else
    hipLaunchKernelGGL(csr_tile_index_kernel<false>, grid, dim3(kBlock), 0, s, p.rowptr, p.col, p.n_rows, p.tile_index,
                       csr_tiles(d), csr_tile_shift(d));
  return hipGetLastError();
}

namespace {

// Tiles per workgroup of the pipelined gradient pass: 4.89 ms per iteration at 8, 4.81 at 16, 4.78 at 32
// (d = 2^24, 64 workers, minibatch 512; 5.18 ms with one tile per workgroup).
constexpr uint32_t kCsrRun = 16;

template <bool PAIRS>
hipError_t csr_grad_launches(const LogregData& p, uint64_t d, uint32_t M, uint32_t batch, float l2, const uint32_t* idx,
                             int64_t* rowbase, uint32_t* bounds, float* zpart, float* z, const float* w, float* g,
                             const ScaleFusion* fuse, uint32_t* fused_rows, hipStream_t s) {
  const float inv_b = 1.0f / (float)batch;
  const uint32_t shift = csr_tile_shift(d);
  const uint32_t ntiles = csr_tiles(d);
  const size_t lds_w = sizeof(float) << shift, lds_g = sizeof(double) << shift;
  {  // the g tile exceeds the 64 KiB default limit of dynamic LDS: raised once per device
    static std::mutex attr_mutex;
    static bool attr_done[64] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> attr_lock(attr_mutex);
    if (!attr_done[dev]) {
      const int lds_double = (int)(sizeof(double) << kCsrTileShift);
      const void* big_lds[] = {reinterpret_cast<const void*>(csr_grad_kernel<false, PAIRS>),
                               reinterpret_cast<const void*>(csr_grad_kernel<true, PAIRS>),
                               reinterpret_cast<const void*>(csr_grad_run_kernel<PAIRS, kNormNone>),
                               reinterpret_cast<const void*>(csr_grad_run_kernel<PAIRS, kNormSub>),
                               reinterpret_cast<const void*>(csr_grad_run_kernel<PAIRS, kNormQuot>),
                               reinterpret_cast<const void*>(csr_grad_run_kernel<PAIRS, kNormComb>),
                               reinterpret_cast<const void*>(csr_grad_workers_kernel<PAIRS, kNormNone>),
                               reinterpret_cast<const void*>(csr_grad_workers_kernel<PAIRS, kNormSub>),
                               reinterpret_cast<const void*>(csr_grad_workers_kernel<PAIRS, kNormQuot>),
                               reinterpret_cast<const void*>(csr_z_wide_kernel<PAIRS>)};
      const int bytes[] = {lds_double, lds_double, lds_double, lds_double, lds_double, lds_double, lds_double,
                           lds_double, lds_double, (int)(2 * sizeof(float) << kCsrTileShift)};
      for (int k = 0; k < 10; ++k) {
        const hipError_t e = hipFuncSetAttribute(big_lds[k], hipFuncAttributeMaxDynamicSharedMemorySize, bytes[k]);
        if (e != hipSuccess) return e;
      }
      attr_done[dev] = true;
    }
  }
  if (p.tile_index != nullptr) {
    dim3 grid((ntiles + 1 + kGatherTile - 1) / kGatherTile, (batch + kGatherTile - 1) / kGatherTile, M);
    hipLaunchKernelGGL(csr_gather_bounds_kernel, grid, dim3(kBlock), 0, s, p.rowptr, p.tile_index, idx, rowbase, bounds,
                       batch, ntiles);
  } else {
    hipLaunchKernelGGL(csr_bounds_kernel<PAIRS>, dim3(batch, M), dim3(kBlock), 0, s, p.rowptr, p.col, idx, rowbase, bounds,
                       batch, ntiles, shift);
  }
  uint32_t nparts = ntiles;  // partial dot products per row
  if (shift == kCsrTileShift && ntiles >= 2) {
    nparts = (ntiles + 1) / 2;
    uint32_t wpb = 1;  // workers per workgroup while 1024 workgroups remain (per iteration at d = 2^24, 64 workers:
                       // 4.538 ms with 8 per workgroup, 4.531 with 16, 4.519 with 32)
    while (wpb < 32 && wpb * 2 <= M && (uint64_t)nparts * (M / (wpb * 2)) >= 1024) wpb *= 2;
    hipLaunchKernelGGL(csr_z_wide_kernel<PAIRS>, dim3(nparts, (M + wpb - 1) / wpb), dim3(kCsrThreads), 2 * lds_w, s, p.col,
                       p.val, rowbase, bounds, w, zpart, d, batch, ntiles, nparts, M, wpb);
  } else {
    hipLaunchKernelGGL(csr_z_kernel<PAIRS>, dim3(M, ntiles), dim3(kCsrThreads), lds_w, s, p.col, p.val, rowbase, bounds, w,
                       zpart, d, batch, ntiles, shift);
  }
  hipLaunchKernelGGL(csr_z_reduce_kernel, dim3((batch + kReduceRows - 1) / kReduceRows, M), dim3(kBlock), 0, s, zpart, p.y, idx,
                     z, batch, nparts, inv_b);
  // The scale pass rides along when every tile is a full one and the write-out is the plain one.
  if (fuse != nullptr && fused_rows != nullptr && shift == kCsrTileShift && d % (1ull << kCsrTileShift) == 0 &&
      l2 == 0.f && ntiles <= kAbsmaxMaxBlocks && aligned16(g) && aligned16(fuse->gref) && aligned16(fuse->gref2)) {
    // (the combined form keeps two references per column: they do not fit next to the pipeline's registers)
    if (batch <= (uint32_t)kCsrRows && M >= 2 && fuse->norm != kNormComb) {
      // a workgroup per tile and group of workers: groups as long as 1024 workgroups (four per compute unit)
      // remain -- per iteration at d = 2^24, 64 workers: 4.69 ms with groups of 8, 4.61 with 16, 4.57 with
      // 32, 4.54 with all 64 (4.76 with the kernel that runs over tiles)
      uint32_t per_group = 64;
      while (per_group > 2 && (uint64_t)ntiles * ((M + per_group - 1) / per_group) < 1024) per_group /= 2;
      const dim3 grid(ntiles, (M + per_group - 1) / per_group);
#define TNG_WORKERS(NORM)                                                                                              \
  hipLaunchKernelGGL((csr_grad_workers_kernel<PAIRS, NORM>), grid, dim3(kCsrThreads), lds_g, s, p.col, p.val, rowbase, \
                     bounds, z, g, d, batch, ntiles, M, per_group, *fuse)
      switch (fuse->norm) {
        case kNormSub: TNG_WORKERS(kNormSub); break;
        case kNormQuot: TNG_WORKERS(kNormQuot); break;
        default: TNG_WORKERS(kNormNone); break;
      }
#undef TNG_WORKERS
    } else if (batch <= (uint32_t)kCsrRows) {
      const uint32_t run = kCsrRun;
      const dim3 grid(M, (ntiles + run - 1) / run);
#define TNG_RUN(NORM)                                                                                                   \
  hipLaunchKernelGGL((csr_grad_run_kernel<PAIRS, NORM>), grid, dim3(kCsrThreads), lds_g, s, p.col, p.val, rowbase, bounds, \
                     z, g, d, batch, ntiles, *fuse)
      switch (fuse->norm) {
        case kNormSub: TNG_RUN(kNormSub); break;
        case kNormQuot: TNG_RUN(kNormQuot); break;
        case kNormComb: TNG_RUN(kNormComb); break;
        default: TNG_RUN(kNormNone); break;
      }
#undef TNG_RUN
    } else {
      hipLaunchKernelGGL((csr_grad_kernel<true, PAIRS>), dim3(M, ntiles), dim3(kCsrThreads), lds_g, s, p.col, p.val,
                         rowbase, bounds, z, w, g, d, batch, ntiles, shift, l2, *fuse);
    }
    *fused_rows = ntiles;
  } else {
    hipLaunchKernelGGL((csr_grad_kernel<false, PAIRS>), dim3(M, ntiles), dim3(kCsrThreads), lds_g, s, p.col, p.val, rowbase,
                       bounds, z, w, g, d, batch, ntiles, shift, l2, ScaleFusion{});
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_logreg_csr_grad(const LogregData& p, uint64_t d, uint32_t M, uint32_t batch, float l2,
                                  const uint32_t* idx, int64_t* rowbase, uint32_t* bounds, float* zpart, float* z,
                                  const float* w, float* g, const ScaleFusion* fuse, uint32_t* fused_rows,
                                  hipStream_t s) {
  if (fused_rows != nullptr) *fused_rows = 0;
  return p.pairs ? csr_grad_launches<true>(p, d, M, batch, l2, idx, rowbase, bounds, zpart, z, w, g, fuse, fused_rows, s)
                 : csr_grad_launches<false>(p, d, M, batch, l2, idx, rowbase, bounds, zpart, z, w, g, fuse, fused_rows, s);
}

hipError_t launch_rosenbrock_grad(uint64_t d, uint32_t M, const float* x, const float* noise, NoiseGen gen, float* g,
                                  const ScaleFusion* fuse, uint32_t* fused_rows, hipStream_t s) {
  if (fused_rows != nullptr) *fused_rows = 0;
  if (d >= 4 && aligned16(x)) {
    const uint64_t nvec = d / 4;
    const uint32_t blocks = (uint32_t)((nvec + kBlock - 1) / kBlock);
    // the fused scale pass sees the vector part only, so it needs all of d there
    if (d % 4 == 0 && fuse != nullptr && fused_rows != nullptr && blocks <= kAbsmaxMaxBlocks && aligned16(fuse->gref) &&
        aligned16(fuse->gref2)) {
      hipLaunchKernelGGL(rosenbrock_vec_kernel<true>, dim3(blocks), dim3(kBlock), 0, s, x, noise, gen, g, d, M, *fuse);
      *fused_rows = blocks;
    } else {
      hipLaunchKernelGGL(rosenbrock_vec_kernel<false>, dim3(blocks), dim3(kBlock), 0, s, x, noise, gen, g, d, M,
                         ScaleFusion{});
    }
    if (d % 4 != 0)  // the last d mod 4 coordinates
      hipLaunchKernelGGL(rosenbrock_kernel, dim3(1), dim3(kBlock), 0, s, x, noise, gen, g, 4 * nvec, d, M);
    return hipGetLastError();
  }
  const uint64_t bx = (d + kBlock - 1) / kBlock;
  hipLaunchKernelGGL(rosenbrock_kernel, dim3((uint32_t)(bx < 16384 ? bx : 16384)), dim3(kBlock), 0, s, x, noise, gen,
                     g, (uint64_t)0, d, M);
  return hipGetLastError();
}

}  // namespace tng
