// The four linear projections of the incremental listings (paper Section 2.4
// and Section 3): q = einsum('bd,hdk->bhk'), the new K / V rows
// einsum('bd,dk->bk') (multi-head: 'bd,hdk->bhk') and y = einsum('bhv,hdv->bd').
// float32 in, float32 products and accumulation on the matrix cores
// (v_mfma_f32_32x32x2_f32), float32 out.
//
// All four are one GEMM out[rows, N] = in[rows, C] . B[C, N] with B addressed
// inside the projection tensor P [h, d, kv]:
//   Q / KV / KV_MH : C = d,    N = h*kv, B[t, n]  = P[n/kv][t][n%kv]   (N contiguous)
//   O              : C = h*kv, N = d,    B[c, t]  = P[c/kv][t][c%kv]   (C contiguous)
//
// One workgroup of 8 waves per 32x32 (or, for small GEMMs, 16x16) output tile.  The
// contraction axis is cut into groups of 4 chunks of 8 (16); wave w takes groups w, w+8, ... (one group in
// flight while the previous one is multiplied) and the eight partial tiles are
// summed through LDS.  With at most a few hundred rows these GEMMs are
// bound by the fp32 matrix rate and by launch latency, not by HBM, so operands
// are read straight from global memory (L2-resident) in MFMA layout:
//   A operand: lane (i, kk) holds in[row0+i][c0 + 4kk + e], e = 0..3 (one 16-byte load),
//              and MFMA e of the chunk contracts slots {c0+e, c0+4+e};
//   B operand: lane (kk, j) holds B[c0 + 4kk + e][n0+j]: four 4-byte loads when N is
//              contiguous, one 16-byte load when C is.
#include "common.hpp"

namespace mqa {
namespace {

typedef __attribute__((ext_vector_type(16))) float floatx16;
typedef __attribute__((ext_vector_type(4))) float floatx4;

constexpr int NWAVES = 8;
constexpr int GC = 4;        // chunks of contraction indices fetched together

// One T x T output tile of out = in . B, left as NWAVES partial tiles in `red` (the caller sums
// them after the barrier this function ends with).  B is addressed inside P [h, C or N, kv]; n0
// is the tile's first column (OUT_PROJ: of d; else of h*kv), rows / columns past the end are
// clamped to the last one and must be discarded by the caller.
template <bool OUT_PROJ, int T, int RB>
__device__ __forceinline__ void gemm_tile(const float* __restrict__ in, const float* __restrict__ P,
                                          int rows, int d, int h, int kv, int row0, int n0,
                                          float (*red)[RB * T * T]) {
  constexpr int TN = T;
  constexpr int CH = 256 / T;                  // contraction indices per chunk (4 per lane group)
  constexpr int NACC = T * T / 64;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i32 = lane % T, kk = lane / T;
  const int C = OUT_PROJ ? h * kv : d;
  const int N = OUT_PROJ ? d : h * kv;
  const size_t head_stride = (size_t)d * kv;

  // A: this lane's row in each of the RB row blocks (clamped; rows past the end are discarded at the store)
  const float* arow[RB];
#pragma unroll
  for (int r = 0; r < RB; ++r) arow[r] = in + (size_t)min(row0 + r * T + i32, rows - 1) * C + 4 * kk;
  // B: this lane's output column n = n0 + i32 (clamped likewise); shared by the row blocks
  const int n = min(n0 + i32, N - 1);
  const float* bcol;       // OUT_PROJ: contiguous along c;  else: element (t, n), stride kv along t
  if (OUT_PROJ) bcol = P + (size_t)n * kv + 4 * kk;                      // + (c / kv) * head_stride + c % kv
  else bcol = P + (size_t)(n / kv) * head_stride + (n % kv) + (size_t)(4 * kk) * kv;

  typedef __attribute__((ext_vector_type(NACC))) float accv;
  accv acc[RB];
#pragma unroll
  for (int r = 0; r < RB; ++r)
#pragma unroll
    for (int e = 0; e < NACC; ++e) acc[r][e] = 0.f;

  const int nchunks = C / CH;                  // C is a multiple of 8; a last half chunk (T = 16) is handled below
  const int tail = C - nchunks * CH;           // 0 or 8 (only when T = 16)
  const int ngroups = (nchunks + (tail ? 1 : 0) + GC - 1) / GC;
  auto load_group = [&](int grp, float4 (&a)[RB][GC], float4 (&b)[GC]) {
#pragma unroll
    for (int e = 0; e < GC; ++e) {
      const int chunk = grp * GC + e;
      // the last, half-filled chunk of a 16-wide contraction: only lane groups kk < 2 hold data
      if (chunk < nchunks || (chunk == nchunks && tail && kk < 2)) {
        const int c0 = chunk * CH;
#pragma unroll
        for (int r = 0; r < RB; ++r) a[r][e] = *reinterpret_cast<const float4*>(arow[r] + c0);
        if (OUT_PROJ) {
          const int c = c0 + 4 * kk;                 // 4 consecutive c stay inside one head (kv % 8 == 0)
          b[e] = *reinterpret_cast<const float4*>(P + (size_t)(c / kv) * head_stride + (size_t)n * kv + (c % kv));
        } else {
          const float* bp = bcol + (size_t)c0 * kv;
          b[e] = make_float4(bp[0], bp[kv], bp[2 * (size_t)kv], bp[3 * (size_t)kv]);
        }
      } else {
#pragma unroll
        for (int r = 0; r < RB; ++r) a[r][e] = make_float4(0.f, 0.f, 0.f, 0.f);
        b[e] = make_float4(0.f, 0.f, 0.f, 0.f);
      }
    }
  };
  auto multiply = [&](const float4 (&a)[RB][GC], const float4 (&b)[GC]) {
#pragma unroll
    for (int e = 0; e < GC; ++e)
#pragma unroll
      for (int r = 0; r < RB; ++r) {
        if constexpr (T == 32) {
          acc[r] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[r][e].x, b[e].x, acc[r], 0, 0, 0);
          acc[r] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[r][e].y, b[e].y, acc[r], 0, 0, 0);
          acc[r] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[r][e].z, b[e].z, acc[r], 0, 0, 0);
          acc[r] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[r][e].w, b[e].w, acc[r], 0, 0, 0);
        } else {
          acc[r] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[r][e].x, b[e].x, acc[r], 0, 0, 0);
          acc[r] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[r][e].y, b[e].y, acc[r], 0, 0, 0);
          acc[r] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[r][e].z, b[e].z, acc[r], 0, 0, 0);
          acc[r] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[r][e].w, b[e].w, acc[r], 0, 0, 0);
        }
      }
  };

  float4 a0[RB][GC], b0[GC], a1[RB][GC], b1[GC];
  int grp = wave;
  if (grp < ngroups) load_group(grp, a0, b0);
  while (grp < ngroups) {
    if (grp + NWAVES < ngroups) load_group(grp + NWAVES, a1, b1);
    multiply(a0, b0);
    grp += NWAVES;
    if (grp >= ngroups) break;
    if (grp + NWAVES < ngroups) load_group(grp + NWAVES, a0, b0);
    multiply(a1, b1);
    grp += NWAVES;
  }

  // D layout: register e of lane (j, g) is tile element (8*(e/4) + 4*g + e%4, j) for the 32x32
  // tile and (4*g + e, j) for the 16x16 tile; row block r adds r*T rows
#pragma unroll
  for (int r = 0; r < RB; ++r)
#pragma unroll
    for (int e = 0; e < NACC; ++e) {
      const int trow = r * T + ((T == 32) ? (8 * (e >> 2) + 4 * kk + (e & 3)) : (4 * kk + e));
      red[wave][trow * TN + i32] = acc[r][e];
    }
  __syncthreads();
}

__device__ __forceinline__ float sum_partials(const float* red0, int e, int stride) {
  return ((red0[e] + red0[stride + e]) + (red0[2 * stride + e] + red0[3 * stride + e])) +
         ((red0[4 * stride + e] + red0[5 * stride + e]) + (red0[6 * stride + e] + red0[7 * stride + e]));
}

// T = 32: 32x32 tiles (v_mfma_f32_32x32x2_f32, chunks of 8 contraction indices);
// T = 16: 16x16 tiles (v_mfma_f32_16x16x4_f32, chunks of 16) for GEMMs too small to fill the
// chip with 32x32 tiles.  Lane (i, kk): i = lane % T, kk = lane / T.
template <bool OUT_PROJ, int T, int RB>
__global__ __launch_bounds__(NWAVES * 64)
void project_mfma_kernel(const float* __restrict__ in, const float* __restrict__ P, float* out,
                         int rows, int d, int h, int kv, int epilogue) {
  constexpr int TM = RB * T;
  __shared__ float red[NWAVES][TM * T];
  const int N = OUT_PROJ ? d : h * kv;
  const int row0 = blockIdx.y * TM, n0 = blockIdx.x * T;
  gemm_tile<OUT_PROJ, T, RB>(in, P, rows, d, h, kv, row0, n0, red);
  for (int e = threadIdx.x; e < TM * T; e += NWAVES * 64) {
    const int r = e / T, c = e % T;
    if (row0 + r < rows && n0 + c < N) {
      float* dst = out + (size_t)(row0 + r) * N + n0 + c;
      *dst = apply_epilogue(sum_partials(&red[0][0], e, TM * T), dst, epilogue);
    }
  }
}

template <typename CT> __device__ __forceinline__ CT cache_value(float x);
template <> __device__ __forceinline__ float cache_value<float>(float x) { return x; }
template <> __device__ __forceinline__ uint16_t cache_value<uint16_t>(float x) { return (uint16_t)float_to_bf16_rne(x); }

// The first three lines of the incremental listings in one launch: q = x . P_q to memory, the
// new K and V rows x . P_k, x . P_v straight into row lens_in[i] of the caches (rounded to the
// cache type), and lens_out[i] = lens_in[i] + 1.  Column tiles are numbered over q's h*k
// columns, then K's h_kv*k, then V's h_kv*v (k and v are multiples of T, so a tile belongs to
// one of them).  A sequence at capacity keeps its cache and its length.
template <int T, int RB, typename CT>
__global__ __launch_bounds__(NWAVES * 64)
void project_qkv_append_kernel(const float* __restrict__ x, const float* __restrict__ P_q,
                               const float* __restrict__ P_k, const float* __restrict__ P_v,
                               float* __restrict__ q, CT* __restrict__ K, CT* __restrict__ V,
                               const int32_t* __restrict__ lens_in, int32_t* __restrict__ lens_out,
                               int rows, int d, int h, int h_kv, int cap, int k, int v) {
  constexpr int TM = RB * T;
  __shared__ float red[NWAVES][TM * T];
  const int row0 = blockIdx.y * TM;
  int n0 = blockIdx.x * T;
  const int nq = h * k, nk = h_kv * k;
  int which = 0;                       // 0: q, 1: K row, 2: V row
  if (n0 >= nq + nk) { which = 2; n0 -= nq + nk; }
  else if (n0 >= nq) { which = 1; n0 -= nq; }
  const int kv = which == 2 ? v : k;
  gemm_tile<false, T, RB>(x, which == 0 ? P_q : which == 1 ? P_k : P_v, rows, d, which == 0 ? h : h_kv, kv, row0, n0, red);
  for (int e = threadIdx.x; e < TM * T; e += NWAVES * 64) {
    const int r = e / T, c = e % T;
    const int row = row0 + r, n = n0 + c;
    if (row >= rows) continue;
    const float val = sum_partials(&red[0][0], e, TM * T);
    if (which == 0) {
      q[(size_t)row * nq + n] = val;
    } else {
      const int L = lens_in[row];
      if (L < 0 || L >= cap) continue;
      CT* dst = which == 1 ? K : V;
      dst[(((size_t)row * h_kv + n / kv) * cap + L) * kv + (n % kv)] = cache_value<CT>(val);
    }
  }
  if (blockIdx.x == 0 && threadIdx.x < TM && row0 + threadIdx.x < rows) {
    const int L = lens_in[row0 + threadIdx.x];
    lens_out[row0 + threadIdx.x] = (L < 0 || L >= cap) ? L : L + 1;
  }
}

}  // namespace

// Tile choice for the split-contraction kernel: 64x32 tiles (two 32x32 blocks sharing the weight
// operand) when there are at least 256 of them (a workgroup per CU), else 32x32 tiles likewise; else, for long contractions, 32x16 tiles (two 16x16 blocks sharing the weight
// operand: a quarter fewer L1 accesses per MFMA; measured 30 -> 26 us at C = 4096 but 9.4 -> 11.4 us
// at C = 1024, where the launch is latency-bound and more workgroups help) when there are at least
// 256 of those; else 16x16 tiles.
enum TileKind { kTile64x32, kTile32, kTile32x16, kTile16 };
static TileKind pick_tile(long long ncols, int rows, int C) {
  if (((ncols + 31) / 32) * ((rows + 63) / 64) >= 256) return kTile64x32;
  if (((ncols + 31) / 32) * ((rows + 31) / 32) >= 256) return kTile32;
  if (C >= 2048 && ((ncols + 15) / 16) * ((rows + 31) / 32) >= 256) return kTile32x16;
  return kTile16;
}

hipError_t launch_project(int mode, const float* in, const float* P, float* out,
                          int rows, int d, int h, int kv, int epilogue, hipStream_t st) {
  const hipError_t big = launch_gemm_tiled(mode, in, P, out, rows, d, h, kv, epilogue, st);     // large GEMMs: LDS-tiled kernel
  if (big != hipErrorNotSupported) return big;
  const bool outp = (mode == 3);
  const int N = outp ? d : h * kv;
  const dim3 block(NWAVES * 64);
#define MQA_PROJ(T, RB)                                                                                              \
  do {                                                                                                               \
    const dim3 grid((N + T - 1) / T, (rows + RB * T - 1) / (RB * T));                                                \
    if (outp) hipLaunchKernelGGL((project_mfma_kernel<true, T, RB>), grid, block, 0, st, in, P, out, rows, d, h, kv, epilogue); \
    else hipLaunchKernelGGL((project_mfma_kernel<false, T, RB>), grid, block, 0, st, in, P, out, rows, d, h, kv, epilogue);     \
  } while (0)
  switch (pick_tile(N, rows, outp ? h * kv : d)) {
    case kTile64x32: MQA_PROJ(32, 2); break;
    case kTile32: MQA_PROJ(32, 1); break;
    case kTile32x16: MQA_PROJ(16, 2); break;
    default: MQA_PROJ(16, 1); break;
  }
#undef MQA_PROJ
  return hipGetLastError();
}

hipError_t launch_project_qkv_append(const float* x, const float* P_q, const float* P_k, const float* P_v,
                                     float* q, void* K, void* V, const int32_t* lens_in, int32_t* lens_out,
                                     int rows, int d, int h, int h_kv, int cap, int k, int v, int is_bf16,
                                     hipStream_t st) {
  const hipError_t big = launch_gemm_tiled_qkv(x, P_q, P_k, P_v, q, K, V, lens_in, lens_out, rows, d, h, h_kv, cap, k, v,
                                               is_bf16, st);
  if (big != hipErrorNotSupported) return big;
  const int ntot = h * k + h_kv * (k + v);
  TileKind kind = pick_tile(ntot, rows, d);
  if ((kind == kTile32 || kind == kTile64x32) && ((k % 32) || (v % 32))) kind = kTile32x16;       // column tiles must not straddle q / K / V
  const dim3 block(NWAVES * 64);
#define MQA_QKV(T, RB)                                                                                               \
  do {                                                                                                               \
    const dim3 grid(ntot / T, (rows + RB * T - 1) / (RB * T));                                                       \
    if (is_bf16) hipLaunchKernelGGL((project_qkv_append_kernel<T, RB, uint16_t>), grid, block, 0, st, x, P_q, P_k, P_v, q, \
                                    (uint16_t*)K, (uint16_t*)V, lens_in, lens_out, rows, d, h, h_kv, cap, k, v);     \
    else hipLaunchKernelGGL((project_qkv_append_kernel<T, RB, float>), grid, block, 0, st, x, P_q, P_k, P_v, q,       \
                            (float*)K, (float*)V, lens_in, lens_out, rows, d, h, h_kv, cap, k, v);                   \
  } while (0)
  switch (kind) {
    case kTile64x32: MQA_QKV(32, 2); break;
    case kTile32: MQA_QKV(32, 1); break;
    case kTile32x16: MQA_QKV(16, 2); break;
    default: MQA_QKV(16, 1); break;
  }
#undef MQA_QKV
  return hipGetLastError();
}

}  // namespace mqa
