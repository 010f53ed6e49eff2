// Generic decode attention: float32 or bf16 cache, any k, v <= 256 (multiples of 8), any
// number of heads, plain float32 FMAs.  Same contract and partial-state format as the MFMA
// kernel; used for float32 caches and for shapes the MFMA kernel does not cover.  One
// workgroup per (KV group, position range); heads are processed in groups of 8, positions in
// tiles of 64 or 128 whose K and V rows are staged in LDS with wide loads all in flight at once
// (these shapes are latency-bound: the point is few dependent round trips, not bandwidth).
//
// Per tile (paper Section 3 incremental listing, lines logits / weights / o):
//   logits[j,p] = sum_c q[j,c] K[p,c]        (q pre-multiplied by scale*log2 e)
//   online softmax state per head: m (max), l (sum of 2^(logit-m)), acc (sum of 2^(logit-m) V[p,:])
#include "common.hpp"

namespace mqa {
namespace {

constexpr int kHeads = 8;     // heads per pass
// positions per tile: TILE = 64, or 128 when k and v are small enough for the LDS (fewer
// dependent round trips per position: these launches are latency-bound)
constexpr int kThreads = 256;

// four consecutive cache elements as floats (row offsets are multiples of 4 elements)
__device__ __forceinline__ float4 load4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ float4 load4(const uint16_t* p) {
  const uint2 u = *reinterpret_cast<const uint2*>(p);
  return make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xffff0000u),
                     __uint_as_float(u.y << 16), __uint_as_float(u.y & 0xffff0000u));
}

// LDS in floats: q rows, the K and V tiles (re-used at the end for the partial outputs of the
// position groups, PG * kHeads * v <= 8192 floats), logits / weights, per-head state.
__host__ __device__ constexpr size_t tile_region_floats(int k, int v, int tile) {
  const size_t tiles = (size_t)tile * (k + 4) + (size_t)tile * v;
  return tiles > 8192 ? tiles : 8192;
}

template <typename T, int TILE>
__global__ __launch_bounds__(kThreads)
void decode_generic_kernel(DecodeParams p) {
  constexpr int kTile = TILE;
  constexpr int HPT = kHeads * kTile / kThreads;      // heads per thread in the logits phase (2 or 4)
  extern __shared__ __align__(16) float smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int k = p.k, v = p.v;
  const int kp = k + 4;                   // K row pitch: keeps float4 alignment, spreads rows over banks
  float* sq = smem;                       // [kHeads][k]
  float* sk = sq + kHeads * k;            // [kTile][k+4]
  float* sv = sk + kTile * kp;            // [kTile][v]
  float* sw = sk + tile_region_floats(k, v, kTile);   // [kHeads][kTile] logits, then weights
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
  // heads of this workgroup: small batches are spread over the chip by giving every workgroup a
  // few heads only (blockIdx.y), each re-reading the sequence's small K/V
  const int hpb = (p.G + p.HG - 1) / p.HG;
  const int hstart = blockIdx.y * hpb, hend = min(p.G, hstart + hpb);
  if (end <= begin) {
    if (p.PS == 0)
      for (int idx = tid; idx < (hend - hstart) * v; idx += kThreads) p.o[((size_t)seq * p.G + hstart) * v + idx] = 0.f;
    return;
  }
  const T* Kseq = reinterpret_cast<const T*>(p.K) + (size_t)seq * p.cap * k;
  const T* Vseq = reinterpret_cast<const T*>(p.V) + (size_t)seq * p.cap * v;
  const int k4 = k >> 2, v4 = v >> 2;
  // weighted sum: thread = (4 output columns c4, position group pg); it adds the positions
  // pg, pg + PG, ... of a tile for all heads, so every V row is read from LDS once
  const int PG = kThreads / v4;
  const int c4 = tid % v4, pg = tid / v4;
  const bool pv_thread = pg < PG;
  // logits: thread = (position, group of HPT heads): every K row is read kHeads / HPT times
  const int dpos = tid % kTile, dhead0 = (tid / kTile) * HPT;

  for (int h0 = hstart; h0 < hend; h0 += kHeads) {
    const int nh = min(kHeads, hend - h0);
    __syncthreads();
    for (int idx = tid; idx < nh * k4; idx += kThreads) {          // 16-byte loads: one round trip for k <= 128
      float4 x = reinterpret_cast<const float4*>(p.q + ((size_t)seq * p.G + h0) * k)[idx];
      x.x *= p.qscale; x.y *= p.qscale; x.z *= p.qscale; x.w *= p.qscale;
      reinterpret_cast<float4*>(sq)[idx] = x;
    }
    if (tid < kHeads) {
      s_m[tid] = -INFINITY;
      s_l[tid] = 0.f;
    }
    float4 acc[kHeads];
#pragma unroll
    for (int j = 0; j < kHeads; ++j) acc[j] = make_float4(0.f, 0.f, 0.f, 0.f);

    for (int p0 = begin; p0 < end; p0 += kTile) {
      const int np = min(kTile, end - p0);
      __syncthreads();
      // stage the tile's K and V rows (contiguous in memory) as float32
      // (batches of 8 K and 8 V loads per thread issued before any is stored: one memory latency per batch)
      const int nk4 = np * k4, nv4 = np * v4;
      for (int base = 0; base < max(nk4, nv4); base += 8 * kThreads) {
        float4 rk[8], rv[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {                 // rows of a tile are contiguous in memory
          const int idx = base + u * kThreads + tid;
          rk[u] = load4(Kseq + (size_t)p0 * k + 4 * (size_t)min(idx, nk4 - 1));
          rv[u] = load4(Vseq + (size_t)p0 * v + 4 * (size_t)min(idx, nv4 - 1));
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int idx = base + u * kThreads + tid;
          if (idx < nk4) {
            const int r = idx / k4, cc = idx - r * k4;
            *reinterpret_cast<float4*>(sk + r * kp + 4 * cc) = rk[u];
          }
          if (idx < nv4) *reinterpret_cast<float4*>(sv + 4 * idx) = rv[u];
        }
      }
      __syncthreads();
      {
        float dot[HPT];
#pragma unroll
        for (int j = 0; j < HPT; ++j) dot[j] = 0.f;
        if (dpos < np) {
          const float4* kr = reinterpret_cast<const float4*>(sk + dpos * kp);
          const float4* qr = reinterpret_cast<const float4*>(sq) + (size_t)dhead0 * k4;   // same address in all lanes of a head group
#pragma unroll 4
          for (int c = 0; c < k4; ++c) {
            const float4 kx = kr[c];
#pragma unroll
            for (int j = 0; j < HPT; ++j) {
              const float4 qx = qr[j * k4 + c];
              dot[j] = fmaf(qx.x, kx.x, fmaf(qx.y, kx.y, fmaf(qx.z, kx.z, fmaf(qx.w, kx.w, dot[j]))));
            }
          }
        }
#pragma unroll
        for (int j = 0; j < HPT; ++j)
          if (dhead0 + j < nh) sw[(dhead0 + j) * kTile + dpos] = dpos < np ? dot[j] : -INFINITY;
      }
      __syncthreads();
      for (int hh = wave; hh < nh; hh += kThreads / 64) {
        float z[kTile / 64];
        float zmax = -INFINITY;
#pragma unroll
        for (int u = 0; u < kTile / 64; ++u) {
          z[u] = sw[hh * kTile + 64 * u + lane];
          zmax = fmaxf(zmax, z[u]);
        }
        const float mold = s_m[hh];
        const float mnew = fmaxf(mold, wave_max(zmax));
        float esum = 0.f;
#pragma unroll
        for (int u = 0; u < kTile / 64; ++u) {
          const float e = __builtin_amdgcn_exp2f(z[u] - mnew);
          sw[hh * kTile + 64 * u + lane] = e;
          esum += e;
        }
        const float sum = wave_sum(esum);
        if (lane == 0) {
          const float alpha = __builtin_amdgcn_exp2f(mold - mnew);
          s_a[hh] = alpha;
          s_l[hh] = s_l[hh] * alpha + sum;
          s_m[hh] = mnew;
        }
      }
      __syncthreads();
      if (pv_thread) {
#pragma unroll
        for (int j = 0; j < kHeads; ++j) {
          const float al = j < nh ? s_a[j] : 0.f;
          acc[j].x *= al; acc[j].y *= al; acc[j].z *= al; acc[j].w *= al;
        }
        const float4* vp = reinterpret_cast<const float4*>(sv) + c4;
#pragma unroll 4
        for (int pos = pg; pos < np; pos += PG) {
          const float4 x = vp[pos * v4];
#pragma unroll
          for (int j = 0; j < kHeads; ++j) {
            const float w = j < nh ? sw[j * kTile + pos] : 0.f;
            acc[j].x = fmaf(w, x.x, acc[j].x); acc[j].y = fmaf(w, x.y, acc[j].y);
            acc[j].z = fmaf(w, x.z, acc[j].z); acc[j].w = fmaf(w, x.w, acc[j].w);
          }
        }
      }
    }
    // sum the position groups through LDS (the tile buffers are free now), normalise, store
    __syncthreads();
    float* red = sk;                                    // [PG][kHeads][v]
    if (pv_thread) {
#pragma unroll
      for (int j = 0; j < kHeads; ++j)
        if (j < nh) reinterpret_cast<float4*>(red + ((size_t)pg * kHeads + j) * v)[c4] = acc[j];
    }
    __syncthreads();
    for (int idx = tid; idx < nh * v4; idx += kThreads) {
      const int hh = idx / v4, cc = idx - hh * v4;
      float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
      for (int g = 0; g < PG; ++g) {
        const float4 x = reinterpret_cast<const float4*>(red + ((size_t)g * kHeads + hh) * v)[cc];
        a.x += x.x; a.y += x.y; a.z += x.z; a.w += x.w;
      }
      if (p.PS == 0) {
        const float inv = 1.0f / s_l[hh];
        a.x *= inv; a.y *= inv; a.z *= inv; a.w *= inv;
        reinterpret_cast<float4*>(p.o + ((size_t)seq * p.G + h0 + hh) * v)[cc] = a;
      } else {
        reinterpret_cast<float4*>(p.part_o + ((((size_t)seq * p.G + h0 + hh) * p.PS) + p.slot0 + srange) * v)[cc] = a;
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

namespace {
size_t generic_lds_bytes(int k, int v, int tile) {
  return ((size_t)kHeads * k + tile_region_floats(k, v, tile) + kHeads * tile + 3 * kHeads) * sizeof(float);
}
}  // namespace

hipError_t launch_decode_generic(const DecodeParams& p, int is_bf16, hipStream_t st) {
  const bool wide = generic_lds_bytes(p.k, p.v, 128) <= 144 * 1024;       // k = v = 128: 133 KiB
  const size_t lds = generic_lds_bytes(p.k, p.v, wide ? 128 : 64);
  const dim3 grid((unsigned)((size_t)p.nseq * p.S), (unsigned)p.HG), block(kThreads);
  void (*kern)(DecodeParams);
  if (wide) kern = is_bf16 ? decode_generic_kernel<uint16_t, 128> : decode_generic_kernel<float, 128>;
  else kern = is_bf16 ? decode_generic_kernel<uint16_t, 64> : decode_generic_kernel<float, 64>;
  if (lds > 64 * 1024) {     // opt in to more than 64 KiB of LDS (largest cases: 133 KiB and, k = v = 256, 142 KiB)
    static bool done[64][4] = {};     // once per device and kernel variant
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = 0;
    const int slot = (wide ? 2 : 0) | (is_bf16 ? 1 : 0);
    if (!done[dev][slot]) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, 144 * 1024);
      if (e != hipSuccess) return e;
      done[dev][slot] = true;
    }
  }
  hipLaunchKernelGGL(kern, grid, block, lds, st, p);
  return hipGetLastError();
}

}  // namespace mqa
