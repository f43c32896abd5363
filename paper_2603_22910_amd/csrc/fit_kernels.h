// Small fp32 kernels of the closed-form predictor fit: the vector operations of a
// conjugate-gradient solve of (X^T X + ridge I) W = X^T C_drop (Sec. "Training
// Details", reconstruction loss).  The matrix products go through the MFMA
// predictor-product kernel (Gram matrices) and the fp32 tile GEMM (G P).
#pragma once
#include "common.h"

namespace echokv {
namespace fit {

constexpr int kDotBlocks = 1024;

// partial[block] = sum over the block's elements of x[i] * y[i]   (summed on the host in double)
__global__ __launch_bounds__(256) void dot_kernel(const float* x, const float* y, int64_t n, float* partial) {
  float acc = 0.f;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256)
    acc = fmaf(x[i], y[i], acc);
  __shared__ float red[4];
  acc = wave_sum(acc, 64);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) partial[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}

// y += alpha * x
__global__ __launch_bounds__(256) void axpy_kernel(float* y, const float* x, float alpha, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256)
    y[i] = fmaf(alpha, x[i], y[i]);
}

// w += alpha * p ; r -= alpha * ap
__global__ __launch_bounds__(256) void step_kernel(float* w, float* r, const float* p, const float* ap,
                                                   float alpha, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    w[i] = fmaf(alpha, p[i], w[i]);
    r[i] = fmaf(-alpha, ap[i], r[i]);
  }
}

// p = r + beta * p
__global__ __launch_bounds__(256) void direction_kernel(float* p, const float* r, float beta, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256)
    p[i] = fmaf(beta, p[i], r[i]);
}

// dst[r, 0:cols) = src[r, col0 : col0 + cols)   (fp32, row pitches ld_dst / ld_src)
__global__ __launch_bounds__(256) void copy_cols_kernel(float* dst, int64_t ld_dst, int dcol0, const float* src,
                                                        int64_t ld_src, int scol0, int rows, int cols) {
  const int64_t n = (int64_t)rows * cols;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const int64_t r = i / cols; const int c = (int)(i % cols);
    dst[r * ld_dst + dcol0 + c] = src[r * ld_src + scol0 + c];
  }
}

__global__ __launch_bounds__(256) void to_bf16_kernel(bf16_t* dst, const float* src, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256)
    dst[i] = f32_to_bf16(src[i]);
}

__global__ __launch_bounds__(256) void fill_kernel(float* dst, float v, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) dst[i] = v;
}

}  // namespace fit
}  // namespace echokv
