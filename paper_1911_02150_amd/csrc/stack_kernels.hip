// Small kernels around the attention step of a decoder-only stack (pre-layernorm residual
// blocks with a ReLU feed-forward, tied token embedding; the model family of the paper's
// Section 4.1).  They exist so that the whole incremental decoding loop of the benchmark
// stack runs in this library; the attention itself is in decode_*.hip and project.hip.
// All float32; one workgroup (256 threads) per row.
#include "common.hpp"

namespace mqa {
namespace {

__device__ __forceinline__ float block_sum(float x, float* red) {
  x = wave_sum(x);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) red[wave] = x;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}

// y = (x - mean) / sqrt(var + eps), gain 1, bias 0 (biased variance over the row)
__global__ __launch_bounds__(256)
void layernorm_kernel(const float* __restrict__ x, float* __restrict__ y, int d, float eps) {
  __shared__ float red[4];
  const float* xr = x + (size_t)blockIdx.x * d;
  float* yr = y + (size_t)blockIdx.x * d;
  float s = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) s += xr[i];
  const float mean = block_sum(s, red) / d;
  float q = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) {
    const float c = xr[i] - mean;
    q += c * c;
  }
  const float rstd = 1.0f / sqrtf(block_sum(q, red) / d + eps);
  for (int i = threadIdx.x; i < d; i += 256) yr[i] = (xr[i] - mean) * rstd;
}

// The same for rows of a multiple of 4 and at most 256 * 4 * NV floats: the row is read once, with
// 16-byte loads all in flight together, and kept in registers for the mean, the centred sum of
// squares and the result (the rows of a decode step are few: the launch is one memory round trip).
template <int NV>
__global__ __launch_bounds__(256)
void layernorm_rows_kernel(const float* __restrict__ x, float* __restrict__ y, int d, float eps) {
  __shared__ float red[4];
  const float4* xr = reinterpret_cast<const float4*>(x + (size_t)blockIdx.x * d);
  float4* yr = reinterpret_cast<float4*>(y + (size_t)blockIdx.x * d);
  const int d4 = d >> 2;
  float4 r[NV];
#pragma unroll
  for (int u = 0; u < NV; ++u) {
    const int i = threadIdx.x + 256 * u;
    r[u] = i < d4 ? xr[i] : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  float s = 0.f;
#pragma unroll
  for (int u = 0; u < NV; ++u) s += (r[u].x + r[u].y) + (r[u].z + r[u].w);
  const float mean = block_sum(s, red) / d;
  float q = 0.f;
#pragma unroll
  for (int u = 0; u < NV; ++u)
    if (threadIdx.x + 256 * u < d4) {
      const float a = r[u].x - mean, b = r[u].y - mean, c = r[u].z - mean, e = r[u].w - mean;
      q += (a * a + b * b) + (c * c + e * e);
    }
  const float rstd = 1.0f / sqrtf(block_sum(q, red) / d + eps);
#pragma unroll
  for (int u = 0; u < NV; ++u) {
    const int i = threadIdx.x + 256 * u;
    if (i < d4) yr[i] = make_float4((r[u].x - mean) * rstd, (r[u].y - mean) * rstd, (r[u].z - mean) * rstd, (r[u].w - mean) * rstd);
  }
}

// x[row] = E[token[row]] + P[pos[row]]; indices outside the tables are clamped (they live on the
// device, so the host cannot reject them)
__global__ __launch_bounds__(256)
void embed_kernel(const int32_t* __restrict__ tokens, const int32_t* __restrict__ pos,
                  const float* __restrict__ E, const float* __restrict__ P, float* __restrict__ x, int d,
                  int vocab, int max_pos) {
  const int tok = min(max(tokens[blockIdx.x], 0), vocab - 1);
  const int at = min(max(pos[blockIdx.x], 0), max_pos - 1);
  const float* e = E + (size_t)tok * d;
  const float* pp = P + (size_t)at * d;
  float* xr = x + (size_t)blockIdx.x * d;
  for (int i = threadIdx.x; i < d; i += 256) xr[i] = e[i] + pp[i];
}

// a += b   /   a = max(a, 0)
__global__ __launch_bounds__(256)
void add_kernel(float* __restrict__ a, const float* __restrict__ b, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) a[i] += b[i];
}
__global__ __launch_bounds__(256)
void relu_kernel(float* __restrict__ a, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) a[i] = fmaxf(a[i], 0.f);
}

// out[row] = index of the largest element of the row, the lowest index among equals.  One
// workgroup of 1024 threads per row, 16-byte loads (rows are 16-byte aligned when n % 4 == 0).
__device__ __forceinline__ void take_better(float& best, int& bi, float v, int i) {
  if (v > best || (v == best && i < bi)) { best = v; bi = i; }
}

__global__ __launch_bounds__(1024)
void argmax_kernel(const float* __restrict__ x, int32_t* __restrict__ out, int n) {
  __shared__ float sv[16];
  __shared__ int si[16];
  const float* xr = x + (size_t)blockIdx.x * n;
  const int tid = threadIdx.x;
  float best = -INFINITY;
  int bi = 0x7fffffff;
  if ((n & 3) == 0) {
    const float4* x4 = reinterpret_cast<const float4*>(xr);
    for (int i = tid; i < (n >> 2); i += 1024) {
      const float4 v = x4[i];
      take_better(best, bi, v.x, 4 * i);
      take_better(best, bi, v.y, 4 * i + 1);
      take_better(best, bi, v.z, 4 * i + 2);
      take_better(best, bi, v.w, 4 * i + 3);
    }
  } else {
    for (int i = tid; i < n; i += 1024) take_better(best, bi, xr[i], i);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) take_better(best, bi, __shfl_xor(best, o), __shfl_xor(bi, o));
  if ((tid & 63) == 0) { sv[tid >> 6] = best; si[tid >> 6] = bi; }
  __syncthreads();
  if (tid < 64) {
    best = tid < 16 ? sv[tid] : -INFINITY;
    bi = tid < 16 ? si[tid] : 0x7fffffff;
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) take_better(best, bi, __shfl_xor(best, o), __shfl_xor(bi, o));
    if (tid == 0) out[blockIdx.x] = bi < n ? bi : 0;      // a row with nothing comparable (all NaN or -inf): index 0
  }
}

}  // namespace

hipError_t launch_layernorm(const float* x, float* y, int rows, int d, float eps, hipStream_t st) {
  if ((d & 3) == 0 && d <= 1024) hipLaunchKernelGGL(layernorm_rows_kernel<1>, dim3(rows), dim3(256), 0, st, x, y, d, eps);
  else if ((d & 3) == 0 && d <= 4096) hipLaunchKernelGGL(layernorm_rows_kernel<4>, dim3(rows), dim3(256), 0, st, x, y, d, eps);
  else hipLaunchKernelGGL(layernorm_kernel, dim3(rows), dim3(256), 0, st, x, y, d, eps);
  return hipGetLastError();
}
hipError_t launch_embed(const int32_t* tokens, const int32_t* pos, const float* E, const float* P, float* x,
                        int rows, int d, int vocab, int max_pos, hipStream_t st) {
  hipLaunchKernelGGL(embed_kernel, dim3(rows), dim3(256), 0, st, tokens, pos, E, P, x, d, vocab, max_pos);
  return hipGetLastError();
}
hipError_t launch_add(float* a, const float* b, size_t n, hipStream_t st) {
  hipLaunchKernelGGL(add_kernel, dim3((unsigned)((n + 1023) / 1024 < 2048 ? (n + 1023) / 1024 : 2048)), dim3(256), 0, st, a, b, n);
  return hipGetLastError();
}
hipError_t launch_relu(float* a, size_t n, hipStream_t st) {
  hipLaunchKernelGGL(relu_kernel, dim3((unsigned)((n + 1023) / 1024 < 2048 ? (n + 1023) / 1024 : 2048)), dim3(256), 0, st, a, n);
  return hipGetLastError();
}
hipError_t launch_argmax(const float* x, int32_t* out, int rows, int n, hipStream_t st) {
  hipLaunchKernelGGL(argmax_kernel, dim3(rows), dim3(1024), 0, st, x, out, n);
  return hipGetLastError();
}

}  // namespace mqa
