// Generic decode attention: float32 or bf16 cache, any k, v <= 256, any number
// of heads, plain float32 FMAs.  Same contract and partial-state format as the
// MFMA kernel; used for float32 caches and for shapes the MFMA kernel does not
// cover.  One workgroup per (KV group, position range); heads are processed in
// groups of 8, positions in tiles of 64 staged through LDS.
//
// Per tile (paper Section 3 incremental listing, lines logits / weights / o):
//   logits[j,p] = sum_c q[j,c] K[p,c]        (q pre-multiplied by scale*log2 e)
//   online softmax state per head: m (max), l (sum of 2^(logit-m)), acc (sum of 2^(logit-m) V[p,:])
#include "common.hpp"

namespace mqa {
namespace {

constexpr int kHeads = 8;     // heads per pass
constexpr int kTile = 64;     // positions per tile
constexpr int kThreads = 256;
constexpr int kMaxDim = 256;
constexpr int kAccPerThread = kHeads * kMaxDim / kThreads;   // 8

template <typename T> __device__ __forceinline__ float to_float(T x);
template <> __device__ __forceinline__ float to_float<float>(float x) { return x; }
template <> __device__ __forceinline__ float to_float<uint16_t>(uint16_t x) { return bf16_bits_to_float(x); }

template <typename T>
__global__ __launch_bounds__(kThreads)
void decode_generic_kernel(DecodeParams p) {
  extern __shared__ __align__(16) float smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int k = p.k, v = p.v, kp = k + 1;
  float* sq = smem;                       // [kHeads][k]
  float* sk = sq + kHeads * k;            // [kTile][k+1]
  float* sw = sk + kTile * kp;            // [kHeads][kTile] logits, then weights
  float* s_m = sw + kHeads * kTile;       // [kHeads]
  float* s_l = s_m + kHeads;              // [kHeads]
  float* s_a = s_l + kHeads;              // [kHeads] rescale factor of the current tile

  const int srange = blockIdx.x % p.S;
  const int seq = blockIdx.x / p.S;
  int L = p.lens[seq / p.lens_div];
  L = L < 0 ? 0 : (L > p.cap ? p.cap : L);
  const int lo = window_lo(L, p.window);                    // local attention: positions [lo, L)
  const int range0 = window_base(L, p.window) + srange * p.chunk;
  const int begin = max(range0, lo);
  const int end = min(range0 + p.chunk, L);
  if (end <= begin) {
    if (p.S == 1)
      for (int idx = tid; idx < p.G * v; idx += kThreads) p.o[(size_t)seq * p.G * v + idx] = 0.f;
    return;
  }
  const T* Kseq = reinterpret_cast<const T*>(p.K) + (size_t)seq * p.cap * k;
  const T* Vseq = reinterpret_cast<const T*>(p.V) + (size_t)seq * p.cap * v;

  for (int h0 = 0; h0 < p.G; h0 += kHeads) {
    const int nh = min(kHeads, p.G - h0);
    __syncthreads();
    for (int idx = tid; idx < nh * k; idx += kThreads)
      sq[idx] = p.q[((size_t)seq * p.G + h0) * k + idx] * p.qscale;
    if (tid < kHeads) {
      s_m[tid] = -INFINITY;
      s_l[tid] = 0.f;
    }
    float acc[kAccPerThread];
#pragma unroll
    for (int i = 0; i < kAccPerThread; ++i) acc[i] = 0.f;

    for (int p0 = begin; p0 < end; p0 += kTile) {
      const int np = min(kTile, end - p0);
      __syncthreads();
      for (int idx = tid; idx < np * k; idx += kThreads) {
        const int r = idx / k, c = idx - r * k;
        sk[r * kp + c] = to_float<T>(Kseq[(size_t)(p0 + r) * k + c]);
      }
      __syncthreads();
      for (int idx = tid; idx < nh * kTile; idx += kThreads) {
        const int hh = idx / kTile, pos = idx % kTile;
        float dot = -INFINITY;
        if (pos < np) {
          dot = 0.f;
          const float* qr = sq + hh * k;
          const float* kr = sk + pos * kp;
          for (int c = 0; c < k; ++c) dot = fmaf(qr[c], kr[c], dot);
        }
        sw[idx] = dot;
      }
      __syncthreads();
      for (int hh = wave; hh < nh; hh += kThreads / 64) {
        const float z = sw[hh * kTile + lane];
        const float mold = s_m[hh];
        const float mnew = fmaxf(mold, wave_max(z));
        const float e = __builtin_amdgcn_exp2f(z - mnew);
        sw[hh * kTile + lane] = e;
        const float sum = wave_sum(e);
        if (lane == 0) {
          const float alpha = __builtin_amdgcn_exp2f(mold - mnew);
          s_a[hh] = alpha;
          s_l[hh] = s_l[hh] * alpha + sum;
          s_m[hh] = mnew;
        }
      }
      __syncthreads();
#pragma unroll
      for (int i = 0; i < kAccPerThread; ++i) {
        const int idx = tid + i * kThreads;
        if (idx < nh * v) {
          const int hh = idx / v, col = idx - hh * v;
          float a = acc[i] * s_a[hh];
          const float* wr = sw + hh * kTile;
          const T* vp = Vseq + (size_t)p0 * v + col;
          for (int pos = 0; pos < np; ++pos) a = fmaf(wr[pos], to_float<T>(vp[(size_t)pos * v]), a);
          acc[i] = a;
        }
      }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kAccPerThread; ++i) {
      const int idx = tid + i * kThreads;
      if (idx < nh * v) {
        const int hh = idx / v, col = idx - hh * v;
        if (p.S == 1) {
          p.o[((size_t)seq * p.G + h0 + hh) * v + col] = acc[i] / s_l[hh];
        } else {
          p.part_o[(((size_t)seq * p.S + srange) * p.G + h0 + hh) * v + col] = acc[i];
        }
      }
    }
    if (p.S > 1 && tid < nh) {
      const size_t pidx = ((size_t)seq * p.S + srange) * p.G + h0 + tid;
      p.part_m[pidx] = s_m[tid];
      p.part_l[pidx] = s_l[tid];
    }
  }
}

}  // namespace

hipError_t launch_decode_generic(const DecodeParams& p, int is_bf16, hipStream_t st) {
  const size_t lds = ((size_t)kHeads * p.k + (size_t)kTile * (p.k + 1) + kHeads * kTile + 3 * kHeads) * sizeof(float);
  const dim3 grid((unsigned)((size_t)p.nseq * p.S)), block(kThreads);
  void (*kern)(DecodeParams) = is_bf16 ? decode_generic_kernel<uint16_t> : decode_generic_kernel<float>;
  if (lds > 64 * 1024) {     // opt in to more than 64 KiB of LDS (largest case: k = 256)
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(kern, grid, block, lds, st, p);
  return hipGetLastError();
}

}  // namespace mqa
