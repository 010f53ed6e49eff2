// Large float32 GEMMs of the projections (prompt-sized row counts, the feed-forward and
// vocabulary matrices of the decoder stack): out[rows, N] = in[rows, C] . B[C, N] with B addressed
// inside the projection tensor P [h, d, kv] exactly as in project.hip.  float32 products and
// accumulation on the matrix cores (v_mfma_f32_32x32x2_f32).
//
// Workgroup tile BM x BN (128 x 128 or 64 x 64) over K-steps of 32, four waves in a 2 x 2
// arrangement, each wave (BM/2) x (BN/2) = RB x CB blocks of 32 x 32.  Tiles go global ->
// registers -> LDS (double buffered, one barrier per K-step; the next tile's global loads are in
// flight while the current one is multiplied).
//
// LDS layouts and MFMA contraction slots.  An MFMA contracts two indices: lane (i, kk) supplies
// A[i][slot kk] and B[slot kk][i].  Which c a slot stands for is free as long as A and B agree;
// the K-step's 16 MFMAs are numbered (u, e), u, e = 0..3, and slot kk of MFMA (u, e) is
// c = 8u + 4kk + e.  So a lane's A values for fixed u are 4 consecutive c: one 16-byte LDS read
// from As[row][c] (pitch 36 floats: 8 consecutive rows hit 8 different 16-byte bank groups).
//   B with c contiguous in memory (the output projection, P_o / tied embedding): staged like A
//   as Bs[n][c], 16-byte reads.
//   B with n contiguous in memory (q, K, V projections, feed-forward): staged as Bs[c][n] (pitch
//   132) with 16-byte writes and read with 4-byte reads, 32 consecutive n per half wave; the rows
//   of the two lane groups kk = 0, 1 are 4 apart = 16 banks apart.
#include "common.hpp"

namespace mqa {
namespace {

typedef __attribute__((ext_vector_type(16))) float floatx16;

constexpr int BK = 32;
constexpr int kAPitch = BK + 4;          // As[row][c], Bs[n][c]

template <int BN> constexpr int b_tile_floats(bool kcontig) { return kcontig ? BN * kAPitch : BK * (BN + 4); }

// B_KCONTIG = false: B[c][n] = P[(n / kv) * d * kv + c * kv + n % kv]   (C = d, N = h * kv)
// B_KCONTIG = true : B[c][n] = P[(c / kv) * d * kv + n * kv + c % kv]   (C = h * kv, N = d)
template <bool B_KCONTIG, int BM, int BN>
__global__ __launch_bounds__(256)
void gemm_tiled_kernel(const float* __restrict__ in, const float* __restrict__ P, float* out,
                       int rows, int d, int h, int kv, int epilogue) {
  constexpr int RB = BM / 64, CB = BN / 64;            // 32x32 blocks per wave in each direction
  constexpr int A_F4 = BM * BK / 4 / 256;              // float4 loads per thread per K-step
  constexpr int B_F4 = BN * BK / 4 / 256;
  constexpr int A_FLOATS = BM * kAPitch;
  constexpr int B_FLOATS = b_tile_floats<BN>(B_KCONTIG);
  constexpr int BPITCH = BN + 4;                       // Bs[c][n]
  extern __shared__ __align__(16) float smem[];
  constexpr int STAGE = A_FLOATS + B_FLOATS;            // one buffer of the double buffer: A tile, then B tile

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i32 = lane & 31, kk = lane >> 5;
  const int row0 = blockIdx.y * BM;
  const int n0 = blockIdx.x * BN;
  const int C = B_KCONTIG ? h * kv : d;
  const int N = B_KCONTIG ? d : h * kv;
  const int wrow = (wave >> 1) * (BM / 2), wcol = (wave & 1) * (BN / 2);
  const size_t head_stride = (size_t)d * kv;

  // ---- global -> register staging.  A (and B when c is contiguous): thread -> (row t/8 + 32 i, c 4 (t%8)).
  const float* a_src[A_F4];
#pragma unroll
  for (int i = 0; i < A_F4; ++i) a_src[i] = in + (size_t)min(row0 + (tid >> 3) + 32 * i, rows - 1) * C + 4 * (tid & 7);
  // B: per-thread base pointers (without the c offset)
  const float* b_src[B_F4];
#pragma unroll
  for (int i = 0; i < B_F4; ++i) {
    if (B_KCONTIG) {
      const int n = min(n0 + (tid >> 3) + 32 * i, N - 1);
      b_src[i] = P + (size_t)n * kv;                                         // + (c / kv) * head_stride + c % kv
    } else {
      // thread -> (c = t / (BN/4) + (1024/BN) i, n = 4 (t % (BN/4)))
      const int n = min(n0 + 4 * (tid % (BN / 4)), N - 4);
      b_src[i] = P + (size_t)(n / kv) * head_stride + (n % kv);              // + c * kv
    }
  }
  float4 ra[A_F4], rb[B_F4];
  auto load_global = [&](int c0) {
    const int ca = c0 + 4 * (tid & 7);
#pragma unroll
    for (int i = 0; i < A_F4; ++i)
      ra[i] = ca < C ? *reinterpret_cast<const float4*>(a_src[i] + c0) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int i = 0; i < B_F4; ++i) {
      if (B_KCONTIG) {
        rb[i] = ca < C ? *reinterpret_cast<const float4*>(b_src[i] + (size_t)(ca / kv) * head_stride + (ca % kv))
                       : make_float4(0.f, 0.f, 0.f, 0.f);
      } else {
        const int c = c0 + tid / (BN / 4) + (1024 / BN) * i;
        rb[i] = c < C ? *reinterpret_cast<const float4*>(b_src[i] + (size_t)c * kv) : make_float4(0.f, 0.f, 0.f, 0.f);
      }
    }
  };
  auto store_lds = [&](int buf) {
    float* Asb = smem + buf * STAGE;
    float* Bsb = Asb + A_FLOATS;
#pragma unroll
    for (int i = 0; i < A_F4; ++i)
      *reinterpret_cast<float4*>(Asb + ((tid >> 3) + 32 * i) * kAPitch + 4 * (tid & 7)) = ra[i];
#pragma unroll
    for (int i = 0; i < B_F4; ++i) {
      if (B_KCONTIG)
        *reinterpret_cast<float4*>(Bsb + ((tid >> 3) + 32 * i) * kAPitch + 4 * (tid & 7)) = rb[i];
      else
        *reinterpret_cast<float4*>(Bsb + (tid / (BN / 4) + (1024 / BN) * i) * BPITCH + 4 * (tid % (BN / 4))) = rb[i];
    }
  };

  floatx16 acc[RB][CB];
#pragma unroll
  for (int r = 0; r < RB; ++r)
#pragma unroll
    for (int c = 0; c < CB; ++c)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[r][c][e] = 0.f;

  const int nk = (C + BK - 1) / BK;
  load_global(0);
  store_lds(0);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    const float* Asb = smem + buf * STAGE;
    const float* Bsb = Asb + A_FLOATS;
    if (kt + 1 < nk) load_global((kt + 1) * BK);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      float4 a[RB];
      float b[CB][4];
#pragma unroll
      for (int r = 0; r < RB; ++r)
        a[r] = *reinterpret_cast<const float4*>(Asb + (wrow + 32 * r + i32) * kAPitch + 8 * u + 4 * kk);
#pragma unroll
      for (int c = 0; c < CB; ++c) {
        if (B_KCONTIG) {
          const float4 t = *reinterpret_cast<const float4*>(Bsb + (wcol + 32 * c + i32) * kAPitch + 8 * u + 4 * kk);
          b[c][0] = t.x; b[c][1] = t.y; b[c][2] = t.z; b[c][3] = t.w;
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) b[c][e] = Bsb[(8 * u + 4 * kk + e) * BPITCH + wcol + 32 * c + i32];
        }
      }
#pragma unroll
      for (int r = 0; r < RB; ++r)
#pragma unroll
        for (int c = 0; c < CB; ++c) {
          acc[r][c] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[r].x, b[c][0], acc[r][c], 0, 0, 0);
          acc[r][c] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[r].y, b[c][1], acc[r][c], 0, 0, 0);
          acc[r][c] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[r].z, b[c][2], acc[r][c], 0, 0, 0);
          acc[r][c] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[r].w, b[c][3], acc[r][c], 0, 0, 0);
        }
    }
    if (kt + 1 < nk) store_lds(buf ^ 1);
    __syncthreads();
  }

  // D layout of the 32x32 tile: register e of lane (j, g) is element (8 (e/4) + 4 g + e%4, j)
#pragma unroll
  for (int r = 0; r < RB; ++r)
#pragma unroll
    for (int c = 0; c < CB; ++c) {
      const int n = n0 + wcol + 32 * c + i32;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int row = row0 + wrow + 32 * r + 8 * (e >> 2) + 4 * kk + (e & 3);
        if (row >= rows || n >= N) continue;
        float* dst = out + (size_t)row * N + n;
        *dst = apply_epilogue(acc[r][c][e], dst, epilogue);
      }
    }
}

template <bool KC, int BM, int BN>
hipError_t launch_tiled(const float* in, const float* P, float* out, int rows, int d, int h, int kv, int N,
                        int epilogue, hipStream_t st) {
  constexpr size_t lds = 2 * (size_t)(BM * kAPitch + b_tile_floats<BN>(KC)) * sizeof(float);
  auto kern = gemm_tiled_kernel<KC, BM, BN>;
  if (lds > 64 * 1024) {
    static bool done[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = 0;
    if (!done[dev]) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (e != hipSuccess) return e;
      done[dev] = true;
    }
  }
  const dim3 grid((N + BN - 1) / BN, (rows + BM - 1) / BM), block(256);
  hipLaunchKernelGGL(kern, grid, block, lds, st, in, P, out, rows, d, h, kv, epilogue);
  return hipGetLastError();
}

}  // namespace

// Returns hipErrorNotSupported when the GEMM is too small for these tiles to fill the chip (the
// caller then uses the split-contraction kernel of project.hip).
hipError_t launch_gemm_tiled(int mode, const float* in, const float* P, float* out,
                             int rows, int d, int h, int kv, int epilogue, hipStream_t st) {
  const bool outp = (mode == 3);
  const int N = outp ? d : h * kv;
  const long long t128 = (long long)((N + 127) / 128) * ((rows + 127) / 128);
  const long long t64 = (long long)((N + 63) / 64) * ((rows + 63) / 64);
  if (N < 64 || rows < 64) return hipErrorNotSupported;
  if (t128 >= 192)
    return outp ? launch_tiled<true, 128, 128>(in, P, out, rows, d, h, kv, N, epilogue, st)
                : launch_tiled<false, 128, 128>(in, P, out, rows, d, h, kv, N, epilogue, st);
  if (t64 >= 256)
    return outp ? launch_tiled<true, 64, 64>(in, P, out, rows, d, h, kv, N, epilogue, st)
                : launch_tiled<false, 64, 64>(in, P, out, rows, d, h, kv, N, epilogue, st);
  return hipErrorNotSupported;
}

}  // namespace mqa
