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

namespace tng {

namespace {

constexpr int kWavesPerBlock = kBlock / kWave;

// Background: index "uniformly sampled" -- idx = (draw * n_rows) >> 32, draws from stream 1.
__global__ __launch_bounds__(kBlock) void minibatch_indices_kernel(uint32_t k0, uint32_t k1, uint32_t iter,
                                                                   uint32_t batch,
                                                                   const uint64_t* __restrict__ n_rows,
                                                                   uint32_t* __restrict__ idx) {
  const uint32_t m = blockIdx.y;
  const uint32_t j = blockIdx.x * kBlock + threadIdx.x;
  if (j >= batch) return;
  const U32x4 r = philox4x32_10(j >> 2, m, iter, 1u, k0, k1);
  const uint32_t lane = j & 3u;
  const uint32_t x = lane == 0 ? r.x : lane == 1 ? r.y : lane == 2 ? r.z : r.w;
  idx[(uint64_t)m * batch + j] = (uint32_t)(((uint64_t)x * n_rows[m]) >> 32);
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

// z_i = x_i . w and r_i = sigma(z_i) - y_i for one minibatch row per workgroup.
template <bool VEC>
__global__ __launch_bounds__(kBlock) void logreg_dense_resid_kernel(const float* const* __restrict__ Xs,
                                                                    const float* const* __restrict__ ys,
                                                                    const uint32_t* __restrict__ idx,
                                                                    const float* __restrict__ w,
                                                                    float* __restrict__ resid, uint64_t d,
                                                                    uint32_t batch) {
  __shared__ float red[kWavesPerBlock];
  const uint32_t m = blockIdx.y, i = blockIdx.x;
  const uint32_t row = idx[(uint64_t)m * batch + i];
  const float* x = Xs[m] + (uint64_t)row * d;
  float acc = 0.f;
  if (VEC) {
    const float4* x4 = reinterpret_cast<const float4*>(x);
    const float4* w4 = reinterpret_cast<const float4*>(w);
    const uint64_t nvec = d / 4;
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
#pragma unroll 4
    for (uint64_t k = threadIdx.x; k < nvec; k += kBlock) {
      const float4 xv = x4[k], wv = w4[k];
      a0 = __builtin_fmaf(xv.x, wv.x, a0);
      a1 = __builtin_fmaf(xv.y, wv.y, a1);
      a2 = __builtin_fmaf(xv.z, wv.z, a2);
      a3 = __builtin_fmaf(xv.w, wv.w, a3);
    }
    acc = (a0 + a1) + (a2 + a3);
  } else {
    for (uint64_t k = threadIdx.x; k < d; k += kBlock) acc = __builtin_fmaf(x[k], w[k], acc);
  }
  const float z = block_sum(acc, red);
  if (threadIdx.x == 0) resid[(uint64_t)m * batch + i] = logistic_residual(z, ys[m][row]);
}

// g_m[k] = (1/B) sum_i r_i X[idx_i][k] + l2 w[k]; a thread owns 4 (VEC) or 1 columns.
template <bool VEC>
__global__ __launch_bounds__(kBlock) void logreg_dense_grad_kernel(const float* const* __restrict__ Xs,
                                                                   const uint32_t* __restrict__ idx,
                                                                   const float* __restrict__ resid,
                                                                   const float* __restrict__ w,
                                                                   float* __restrict__ g, uint64_t d,
                                                                   uint32_t batch, float inv_b, float l2) {
  __shared__ float sR[kBlock];
  __shared__ uint32_t sRow[kBlock];
  const uint32_t m = blockIdx.y;
  const float* X = Xs[m];
  const uint64_t col = (uint64_t)blockIdx.x * kBlock + threadIdx.x;  // float4 (VEC) or float index
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
          const float4 xv = reinterpret_cast<const float4*>(X + (uint64_t)sRow[i] * d)[col];
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
  if (!active) return;
  if (VEC) {
    const float4 wv = reinterpret_cast<const float4*>(w)[col];
    float4 o;
    o.x = __builtin_fmaf(l2, wv.x, acc.x * inv_b);
    o.y = __builtin_fmaf(l2, wv.y, acc.y * inv_b);
    o.z = __builtin_fmaf(l2, wv.z, acc.z * inv_b);
    o.w = __builtin_fmaf(l2, wv.w, acc.w * inv_b);
    reinterpret_cast<float4*>(g + (uint64_t)m * d)[col] = o;
  } else {
    g[(uint64_t)m * d + col] = __builtin_fmaf(l2, w[col], acc.x * inv_b);
  }
}

// CSR: residual of one minibatch row per workgroup (gather w at the row's columns).
__global__ __launch_bounds__(kBlock) void logreg_csr_resid_kernel(const int64_t* const* __restrict__ rowptrs,
                                                                  const int32_t* const* __restrict__ cols,
                                                                  const float* const* __restrict__ vals,
                                                                  const float* const* __restrict__ ys,
                                                                  const uint32_t* __restrict__ idx,
                                                                  const float* __restrict__ w,
                                                                  float* __restrict__ resid, uint32_t batch) {
  __shared__ float red[kWavesPerBlock];
  const uint32_t m = blockIdx.y, i = blockIdx.x;
  const uint32_t row = idx[(uint64_t)m * batch + i];
  const int64_t a = rowptrs[m][row], b = rowptrs[m][row + 1];
  const int32_t* __restrict__ c = cols[m];
  const float* __restrict__ v = vals[m];
  float acc = 0.f;
#pragma unroll 4
  for (int64_t k = a + threadIdx.x; k < b; k += kBlock) acc = __builtin_fmaf(v[k], w[c[k]], acc);
  const float z = block_sum(acc, red);
  if (threadIdx.x == 0) resid[(uint64_t)m * batch + i] = logistic_residual(z, ys[m][row]);
}

// g[m][:] = l2 * w  (start value of the scatter-add below)
__global__ __launch_bounds__(kBlock) void logreg_csr_init_kernel(const float* __restrict__ w,
                                                                 float* __restrict__ g, uint64_t d, float l2) {
  const uint32_t m = blockIdx.y;
  const uint64_t stride = (uint64_t)gridDim.x * kBlock;
  for (uint64_t e = (uint64_t)blockIdx.x * kBlock + threadIdx.x; e < d; e += stride)
    g[(uint64_t)m * d + e] = l2 != 0.f ? l2 * w[e] : 0.f;
}

__global__ __launch_bounds__(kBlock) void logreg_csr_init_vec_kernel(const float4* __restrict__ w4,
                                                                     float4* __restrict__ g4, uint64_t nvec,
                                                                     float l2) {
  const uint32_t m = blockIdx.y;
  const uint64_t stride = (uint64_t)gridDim.x * kBlock;
  for (uint64_t e = (uint64_t)blockIdx.x * kBlock + threadIdx.x; e < nvec; e += stride) {
    float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
    if (l2 != 0.f) {
      const float4 wv = w4[e];
      o = make_float4(l2 * wv.x, l2 * wv.y, l2 * wv.z, l2 * wv.w);
    }
    g4[(uint64_t)m * nvec + e] = o;
  }
}

// g[m][col] += (r_i / B) * val for every stored entry of every minibatch row (hardware fp32 atomics;
// the summation order, hence the last bits of g, vary from run to run).
__global__ __launch_bounds__(kBlock) void logreg_csr_scatter_kernel(const int64_t* const* __restrict__ rowptrs,
                                                                    const int32_t* const* __restrict__ cols,
                                                                    const float* const* __restrict__ vals,
                                                                    const uint32_t* __restrict__ idx,
                                                                    const float* __restrict__ resid,
                                                                    float* __restrict__ g, uint64_t d,
                                                                    uint32_t batch, float inv_b) {
  const uint32_t m = blockIdx.y, i = blockIdx.x;
  const uint32_t row = idx[(uint64_t)m * batch + i];
  const int64_t a = rowptrs[m][row], b = rowptrs[m][row + 1];
  const int32_t* __restrict__ c = cols[m];
  const float* __restrict__ v = vals[m];
  const float r = resid[(uint64_t)m * batch + i] * inv_b;
  float* gm = g + (uint64_t)m * d;
  for (int64_t k = a + threadIdx.x; k < b; k += kBlock) unsafeAtomicAdd(gm + c[k], r * v[k]);
}

// Chain Rosenbrock gradient ("Nonconvex Problems", d-dimensional form) plus per-worker noise.
// Fixed expression tree, one rounding per operation:
//   a = x[i+1] - x[i]*x[i];  t1 = (-400*x[i])*a;  t2 = -2*(1 - x[i])        (i < d-1)
//   b = x[i] - x[i-1]*x[i-1];  t3 = 200*b                                    (i > 0)
//   g = ((t1 + t2) + t3) + noise, absent terms left out.
__global__ __launch_bounds__(kBlock) void rosenbrock_kernel(const float* __restrict__ x,
                                                            const float* __restrict__ noise,
                                                            float* __restrict__ g, uint64_t d, uint32_t M) {
  const uint64_t stride = (uint64_t)gridDim.x * kBlock;
  for (uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x; i < d; i += stride) {
    const float xi = x[i];
    float base = 0.f;
    bool have = false;
    if (i + 1 < d) {
      const float a = x[i + 1] - xi * xi;
      const float t1 = (-400.0f * xi) * a;
      const float t2 = -2.0f * (1.0f - xi);
      base = t1 + t2;
      have = true;
    }
    if (i > 0) {
      const float xp = x[i - 1];
      const float b = xi - xp * xp;
      const float t3 = 200.0f * b;
      base = have ? base + t3 : t3;
    }
    for (uint32_t m = 0; m < M; ++m) {
      const uint64_t o = (uint64_t)m * d + i;
      g[o] = noise != nullptr ? base + noise[o] : base;
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

hipError_t launch_logreg_dense_grad(const LogregData& p, uint64_t d, uint32_t M, uint32_t batch, float l2,
                                    const uint32_t* idx, float* resid, const float* w, float* g,
                                    hipStream_t s) {
  // Shards are required to be 16-byte aligned; rows stay aligned only when d is a multiple of 4.
  const bool vec = d % 4 == 0 && aligned16(w) && aligned16(g);
  const float inv_b = 1.0f / (float)batch;
  dim3 grid_r(batch, M);
  if (vec) {
    hipLaunchKernelGGL((logreg_dense_resid_kernel<true>), grid_r, dim3(kBlock), 0, s, p.X, p.y, idx, w, resid, d,
                       batch);
    dim3 grid_g((uint32_t)((d / 4 + kBlock - 1) / kBlock), M);
    hipLaunchKernelGGL((logreg_dense_grad_kernel<true>), grid_g, dim3(kBlock), 0, s, p.X, idx, resid, w, g, d,
                       batch, inv_b, l2);
  } else {
    hipLaunchKernelGGL((logreg_dense_resid_kernel<false>), grid_r, dim3(kBlock), 0, s, p.X, p.y, idx, w, resid,
                       d, batch);
    dim3 grid_g((uint32_t)((d + kBlock - 1) / kBlock), M);
    hipLaunchKernelGGL((logreg_dense_grad_kernel<false>), grid_g, dim3(kBlock), 0, s, p.X, idx, resid, w, g, d,
                       batch, inv_b, l2);
  }
  return hipGetLastError();
}

hipError_t launch_logreg_csr_grad(const LogregData& p, uint64_t d, uint32_t M, uint32_t batch, float l2,
                                  const uint32_t* idx, float* resid, const float* w, float* g,
                                  hipStream_t s) {
  const float inv_b = 1.0f / (float)batch;
  dim3 grid_r(batch, M);
  hipLaunchKernelGGL(logreg_csr_resid_kernel, grid_r, dim3(kBlock), 0, s, p.rowptr, p.col, p.val, p.y, idx, w,
                     resid, batch);
  if (d % 4 == 0 && aligned16(w) && aligned16(g)) {
    const uint64_t nvec = d / 4;
    const uint64_t bx = (nvec + kBlock - 1) / kBlock;
    dim3 grid_i((uint32_t)(bx < 2048 ? bx : 2048), M);
    hipLaunchKernelGGL(logreg_csr_init_vec_kernel, grid_i, dim3(kBlock), 0, s,
                       reinterpret_cast<const float4*>(w), reinterpret_cast<float4*>(g), nvec, l2);
  } else {
    const uint64_t bx = (d + kBlock - 1) / kBlock;
    dim3 grid_i((uint32_t)(bx < 2048 ? bx : 2048), M);
    hipLaunchKernelGGL(logreg_csr_init_kernel, grid_i, dim3(kBlock), 0, s, w, g, d, l2);
  }
  hipLaunchKernelGGL(logreg_csr_scatter_kernel, grid_r, dim3(kBlock), 0, s, p.rowptr, p.col, p.val, idx, resid,
                     g, d, batch, inv_b);
  return hipGetLastError();
}

hipError_t launch_rosenbrock_grad(uint64_t d, uint32_t M, const float* x, const float* noise, float* g,
                                  hipStream_t s) {
  const uint64_t bx = (d + kBlock - 1) / kBlock;
  hipLaunchKernelGGL(rosenbrock_kernel, dim3((uint32_t)(bx < 16384 ? bx : 16384)), dim3(kBlock), 0, s, x, noise, g,
                     d, M);
  return hipGetLastError();
}

}  // namespace tng
