// The four linear projections of the incremental listings (paper Section 2.4
// and Section 3): q = einsum('bd,hdk->bhk'), the new K / V rows
// einsum('bd,dk->bk') (multi-head: 'bd,hdk->bhk') and y = einsum('bhv,hdv->bd').
// float32 in, float32 FMAs, float32 out.
//
// All four are one GEMM out[rows, N] = in[rows, C] . B[C, N] with B addressed
// inside the projection tensor P [h, d, kv]:
//   Q / KV / KV_MH : C = d,    N = h*kv, B[t, n]  = P[n/kv][t][n%kv]   (N contiguous)
//   O              : C = h*kv, N = d,    B[c, t]  = P[c/kv][t][c%kv]   (C contiguous)
// Tiles of 32 rows x 64 columns, 32-deep slices through LDS, 2x4 outputs per thread.
#include "common.hpp"

namespace mqa {
namespace {

constexpr int BM = 32, BN = 64, BK = 32, NT = 256;

template <bool OUT_PROJ>
__global__ __launch_bounds__(NT)
void project_kernel(const float* __restrict__ in, const float* __restrict__ P, float* __restrict__ out,
                    int rows, int d, int h, int kv) {
  __shared__ float As[BK][BM + 4];
  __shared__ float Bs[BK][BN + 4];
  const int tid = threadIdx.x;
  const int C = OUT_PROJ ? h * kv : d;
  const int N = OUT_PROJ ? d : h * kv;
  const int r0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int ty = tid >> 4, tx = tid & 15;
  float acc[2][4] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
  const size_t head_stride = (size_t)d * kv;

  for (int c0 = 0; c0 < C; c0 += BK) {
    {  // A slice: 32 rows x 32 contraction indices, one float4 per thread, stored transposed
      const int row = tid >> 3, c4 = (tid & 7) * 4;
      float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
      if (r0 + row < rows && c0 + c4 < C)
        a = *reinterpret_cast<const float4*>(in + (size_t)(r0 + row) * C + c0 + c4);
      As[c4 + 0][row] = a.x; As[c4 + 1][row] = a.y; As[c4 + 2][row] = a.z; As[c4 + 3][row] = a.w;
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int idx = tid + i * NT;
      if (!OUT_PROJ) {   // B[t, n]: float4 along n
        const int kk = idx >> 4, n4 = (idx & 15) * 4;
        const int t = c0 + kk, n = n0 + n4;
        float4 b = make_float4(0.f, 0.f, 0.f, 0.f);
        if (t < C && n < N)
          b = *reinterpret_cast<const float4*>(P + (size_t)(n / kv) * head_stride + (size_t)t * kv + (n % kv));
        *reinterpret_cast<float4*>(&Bs[kk][n4]) = b;
      } else {           // B[c, t]: float4 along c, stored transposed
        const int tt = idx >> 3, c4 = (idx & 7) * 4;
        const int t = n0 + tt, c = c0 + c4;
        float4 b = make_float4(0.f, 0.f, 0.f, 0.f);
        if (t < N && c < C)
          b = *reinterpret_cast<const float4*>(P + (size_t)(c / kv) * head_stride + (size_t)t * kv + (c % kv));
        Bs[c4 + 0][tt] = b.x; Bs[c4 + 1][tt] = b.y; Bs[c4 + 2][tt] = b.z; Bs[c4 + 3][tt] = b.w;
      }
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      const float a0 = As[kk][2 * ty], a1 = As[kk][2 * ty + 1];
      const float4 b = *reinterpret_cast<const float4*>(&Bs[kk][4 * tx]);
      acc[0][0] = fmaf(a0, b.x, acc[0][0]); acc[0][1] = fmaf(a0, b.y, acc[0][1]);
      acc[0][2] = fmaf(a0, b.z, acc[0][2]); acc[0][3] = fmaf(a0, b.w, acc[0][3]);
      acc[1][0] = fmaf(a1, b.x, acc[1][0]); acc[1][1] = fmaf(a1, b.y, acc[1][1]);
      acc[1][2] = fmaf(a1, b.z, acc[1][2]); acc[1][3] = fmaf(a1, b.w, acc[1][3]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int r = r0 + 2 * ty + i, n = n0 + 4 * tx;
    if (r < rows && n < N)
      *reinterpret_cast<float4*>(out + (size_t)r * N + n) = make_float4(acc[i][0], acc[i][1], acc[i][2], acc[i][3]);
  }
}

}  // namespace

hipError_t launch_project(int mode, const float* in, const float* P, float* out,
                          int rows, int d, int h, int kv, hipStream_t st) {
  const bool outp = (mode == 3);
  const int N = outp ? d : h * kv;
  const dim3 grid((N + BN - 1) / BN, (rows + BM - 1) / BM), block(NT);
  if (outp)
    hipLaunchKernelGGL(project_kernel<true>, grid, block, 0, st, in, P, out, rows, d, h, kv);
  else
    hipLaunchKernelGGL(project_kernel<false>, grid, block, 0, st, in, P, out, rows, d, h, kv);
  return hipGetLastError();
}

}  // namespace mqa
