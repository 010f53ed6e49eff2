// Generic decode attention: float32 or bf16 cache, any k, v <= 256 (multiples of 8), any
// number of heads, plain float32 FMAs.  Same contract and partial-state format as the MFMA
// kernel; used for float32 caches and for shapes the MFMA kernel does not cover.  One
// workgroup per (KV group, position range); heads are processed in groups of 8, positions in
// tiles of 64 whose K and V rows are staged in LDS with wide loads all in flight at once
// (these shapes are latency-bound: the point is few dependent round trips, not bandwidth).
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
constexpr int kAccPerThread = kHeads * kMaxDim / kThreads / 4;   // float4 outputs per thread (2)

// four consecutive cache elements as floats (row offsets are multiples of 4 elements)
__device__ __forceinline__ float4 load4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ float4 load4(const uint16_t* p) {
  const uint2 u = *reinterpret_cast<const uint2*>(p);
  return make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xffff0000u),
                     __uint_as_float(u.y << 16), __uint_as_float(u.y & 0xffff0000u));
}

template <typename T>
__global__ __launch_bounds__(kThreads)
void decode_generic_kernel(DecodeParams p) {
  extern __shared__ __align__(16) float smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int k = p.k, v = p.v;
  const int kp = k + 4;                   // K row pitch: keeps float4 alignment, spreads rows over banks
  float* sq = smem;                       // [kHeads][k]
  float* sk = sq + kHeads * k;            // [kTile][k+4]
  float* sv = sk + kTile * kp;            // [kTile][v]
  float* sw = sv + kTile * v;             // [kHeads][kTile] logits, then weights
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
    if (p.PS == 0)
      for (int idx = tid; idx < p.G * v; idx += kThreads) p.o[(size_t)seq * p.G * v + idx] = 0.f;
    return;
  }
  const T* Kseq = reinterpret_cast<const T*>(p.K) + (size_t)seq * p.cap * k;
  const T* Vseq = reinterpret_cast<const T*>(p.V) + (size_t)seq * p.cap * v;
  const int k4 = k >> 2, v4 = v >> 2;

  for (int h0 = 0; h0 < p.G; h0 += kHeads) {
    const int nh = min(kHeads, p.G - h0);
    __syncthreads();
    for (int idx = tid; idx < nh * k; idx += kThreads)
      sq[idx] = p.q[((size_t)seq * p.G + h0) * k + idx] * p.qscale;
    if (tid < kHeads) {
      s_m[tid] = -INFINITY;
      s_l[tid] = 0.f;
    }
    float4 acc[kAccPerThread];
#pragma unroll
    for (int i = 0; i < kAccPerThread; ++i) acc[i] = make_float4(0.f, 0.f, 0.f, 0.f);

    for (int p0 = begin; p0 < end; p0 += kTile) {
      const int np = min(kTile, end - p0);
      __syncthreads();
      // stage the tile's K and V rows (contiguous in memory) as float32
      for (int idx = tid; idx < np * k4; idx += kThreads) {
        const int r = idx / k4, c4 = idx - r * k4;
        *reinterpret_cast<float4*>(sk + r * kp + 4 * c4) = load4(Kseq + (size_t)(p0 + r) * k + 4 * c4);
      }
      for (int idx = tid; idx < np * v4; idx += kThreads)
        *reinterpret_cast<float4*>(sv + 4 * idx) = load4(Vseq + (size_t)p0 * v + 4 * idx);
      __syncthreads();
      for (int idx = tid; idx < nh * kTile; idx += kThreads) {
        const int hh = idx / kTile, pos = idx % kTile;
        float dot = -INFINITY;
        if (pos < np) {
          const float4* qr = reinterpret_cast<const float4*>(sq + hh * k);
          const float4* kr = reinterpret_cast<const float4*>(sk + pos * kp);
          float d0 = 0.f, d1 = 0.f, d2 = 0.f, d3 = 0.f;
          for (int c = 0; c < k4; ++c) {
            const float4 a = qr[c], b = kr[c];
            d0 = fmaf(a.x, b.x, d0); d1 = fmaf(a.y, b.y, d1); d2 = fmaf(a.z, b.z, d2); d3 = fmaf(a.w, b.w, d3);
          }
          dot = (d0 + d1) + (d2 + d3);
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
        const int idx = tid + i * kThreads;          // (head, group of 4 columns)
        if (idx < nh * v4) {
          const int hh = idx / v4, c4 = idx - hh * v4;
          const float al = s_a[hh];
          float4 a = make_float4(acc[i].x * al, acc[i].y * al, acc[i].z * al, acc[i].w * al);
          const float* wr = sw + hh * kTile;
          const float4* vp = reinterpret_cast<const float4*>(sv) + c4;
          for (int pos = 0; pos < np; ++pos) {
            const float w = wr[pos];
            const float4 x = vp[pos * v4];
            a.x = fmaf(w, x.x, a.x); a.y = fmaf(w, x.y, a.y); a.z = fmaf(w, x.z, a.z); a.w = fmaf(w, x.w, a.w);
          }
          acc[i] = a;
        }
      }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kAccPerThread; ++i) {
      const int idx = tid + i * kThreads;
      if (idx < nh * v4) {
        const int hh = idx / v4, c4 = idx - hh * v4;
        float4 a = acc[i];
        if (p.PS == 0) {
          const float inv = 1.0f / s_l[hh];
          a.x *= inv; a.y *= inv; a.z *= inv; a.w *= inv;
          reinterpret_cast<float4*>(p.o + ((size_t)seq * p.G + h0 + hh) * v)[c4] = a;
        } else {
          reinterpret_cast<float4*>(p.part_o + ((((size_t)seq * p.G + h0 + hh) * p.PS) + p.slot0 + srange) * v)[c4] = a;
        }
      }
    }
    if (p.PS > 0 && tid < nh) {
      const size_t pidx = ((size_t)seq * p.G + h0 + tid) * p.PS + p.slot0 + srange;
      p.part_m[pidx] = s_m[tid];
      p.part_l[pidx] = s_l[tid];
    }
  }
}

}  // namespace

hipError_t launch_decode_generic(const DecodeParams& p, int is_bf16, hipStream_t st) {
  const size_t lds = ((size_t)kHeads * p.k + (size_t)kTile * (p.k + 4) + (size_t)kTile * p.v + kHeads * kTile +
                      3 * kHeads) * sizeof(float);
  const dim3 grid((unsigned)((size_t)p.nseq * p.S)), block(kThreads);
  void (*kern)(DecodeParams) = is_bf16 ? decode_generic_kernel<uint16_t> : decode_generic_kernel<float>;
  if (lds > 64 * 1024) {     // opt in to more than 64 KiB of LDS (largest case, k = v = 256: 142 KiB)
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 144 * 1024);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(kern, grid, block, lds, st, p);
  return hipGetLastError();
}

}  // namespace mqa
