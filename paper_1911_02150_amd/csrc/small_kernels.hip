// Combine pass of the split softmax, cache append, beam reorder, and the two streaming
// kernels used as bandwidth references.
#include "common.hpp"

namespace mqa {
namespace {

// Merge the partial softmax states of one output row.  With (m_i, l_i, acc_i) the maximum,
// the sum of 2^(logit - m_i) and the un-normalised weighted sum of V rows over range i (this
// is the softmax of the paper's Section 2.1 written over a partition of the positions):
//   M = max_i m_i,  L = sum_i l_i 2^(m_i - M),  o = sum_i acc_i 2^(m_i - M) / L.
// Only ranges that start before the row's length (per segment) were written.
// The slots of a row are fetched B at a time, all loads of a batch issued before any is used
// and independent of the lengths, so a batch costs one memory latency; batches are folded
// into a running (M, L, o) state.  B = 4 covers the usual 2..4 ranges in one batch.
__device__ __forceinline__ int valid_ranges(const CombineSegment& sg, long long row) {
  int L = sg.lens[row / sg.rows_per_len];
  L = L < 0 ? 0 : (L > sg.cap ? sg.cap : L);
  return min(sg.S, (L - window_base(L, sg.window) + sg.chunk - 1) / sg.chunk);
}

template <int B>
__global__ __launch_bounds__(256)
void combine_kernel(CombineParams p) {
  const int v4 = p.v >> 2;
  const size_t total = (size_t)p.rows * v4;
  // workgroups are dispatched round-robin over the 8 XCDs; take the rows whose partial states
  // the same XCD wrote (the decode kernel's workgroup -> sequence mapping), as far as grids agree
  const unsigned nb = gridDim.x, bid = blockIdx.x;
  const unsigned wid = ((nb & 7) == 0) ? (bid & 7) * (nb >> 3) + (bid >> 3) : bid;
  const size_t idx = (size_t)wid * 256 + threadIdx.x;
  if (idx >= total) return;
  const int c4 = (int)(idx % v4);
  const long long row = (long long)(idx / v4);
  const size_t base = (size_t)row * p.PS;
  const int n0 = valid_ranges(p.seg[0], row);
  const int s1 = p.seg[0].S;
  const int n1 = p.nseg > 1 ? valid_ranges(p.seg[1], row) : 0;
  float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
  float M = -INFINITY, lsum = 0.f;
  for (int sb = 0; sb < p.PS; sb += B) {
    float pm[B], pl[B];
    float4 po[B];
#pragma unroll
    for (int j = 0; j < B; ++j) {
      const size_t pi = base + min(sb + j, p.PS - 1);     // in bounds for every j
      pm[j] = p.part_m[pi];
      pl[j] = p.part_l[pi];
      po[j] = reinterpret_cast<const float4*>(p.part_o + pi * p.v)[c4];
    }
    bool ok[B];
    float Mn = M;
#pragma unroll
    for (int j = 0; j < B; ++j) {
      const int sl = sb + j;                              // unwritten slots are skipped, not multiplied by 0
      ok[j] = sl < p.PS && (sl < n0 || (sl >= s1 && sl < s1 + n1));
      if (ok[j]) Mn = fmaxf(Mn, pm[j]);
    }
    if (Mn == -INFINITY) continue;
    const float f0 = __builtin_amdgcn_exp2f(M - Mn);      // 0 while nothing has been folded in yet
    a.x *= f0; a.y *= f0; a.z *= f0; a.w *= f0;
    lsum *= f0;
#pragma unroll
    for (int j = 0; j < B; ++j)
      if (ok[j]) {
        const float f = __builtin_amdgcn_exp2f(pm[j] - Mn);
        a.x += f * po[j].x; a.y += f * po[j].y; a.z += f * po[j].z; a.w += f * po[j].w;
        lsum += f * pl[j];
      }
    M = Mn;
  }
  if (lsum > 0.f) {                                 // no valid position at all: a zero row
    const float inv = 1.0f / lsum;
    a.x *= inv; a.y *= inv; a.z *= inv; a.w *= inv;
  }
  reinterpret_cast<float4*>(p.o + (size_t)row * p.v)[c4] = a;
}

// The same merge for many slots per row (a few long sequences spread over up to 256 ranges):
// one workgroup per output row, thread = (4 columns, slot group sg); a thread folds the slots
// sg, sg + SG, ... in batches of 8 loads, then the SG partial states are folded through LDS.
__global__ __launch_bounds__(256)
void combine_wide_kernel(CombineParams p) {
  __shared__ float s_m[256], s_l[256];
  __shared__ float4 s_a[256];
  const int v4 = p.v >> 2, SG = 256 / v4;
  const int tid = threadIdx.x;
  const int c4 = tid % v4, sgrp = tid / v4;
  const long long row = blockIdx.x;
  const size_t base = (size_t)row * p.PS;
  const int n0 = valid_ranges(p.seg[0], row);
  const int s1 = p.seg[0].S;
  const int n1 = p.nseg > 1 ? valid_ranges(p.seg[1], row) : 0;
  float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
  float M = -INFINITY, lsum = 0.f;
  if (sgrp < SG) {
    for (int sb = sgrp; sb < p.PS; sb += 8 * SG) {
      float pm[8], pl[8];
      float4 po[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const size_t pi = base + min(sb + j * SG, p.PS - 1);
        pm[j] = p.part_m[pi];
        pl[j] = p.part_l[pi];
        po[j] = reinterpret_cast<const float4*>(p.part_o + pi * p.v)[c4];
      }
      float Mn = M;
      bool ok[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int sl = sb + j * SG;
        ok[j] = sl < p.PS && (sl < n0 || (sl >= s1 && sl < s1 + n1));
        if (ok[j]) Mn = fmaxf(Mn, pm[j]);
      }
      if (Mn == -INFINITY) continue;
      const float f0 = __builtin_amdgcn_exp2f(M - Mn);
      a.x *= f0; a.y *= f0; a.z *= f0; a.w *= f0;
      lsum *= f0;
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (ok[j]) {
          const float f = __builtin_amdgcn_exp2f(pm[j] - Mn);
          a.x += f * po[j].x; a.y += f * po[j].y; a.z += f * po[j].z; a.w += f * po[j].w;
          lsum += f * pl[j];
        }
      M = Mn;
    }
  }
  s_m[tid] = M;
  s_l[tid] = lsum;
  s_a[tid] = a;
  __syncthreads();
  if (sgrp == 0) {
    float Mt = -INFINITY;
    for (int g = 0; g < SG; ++g) Mt = fmaxf(Mt, s_m[g * v4 + c4]);
    float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
    float lt = 0.f;
    if (Mt != -INFINITY)
      for (int g = 0; g < SG; ++g) {
        const float f = __builtin_amdgcn_exp2f(s_m[g * v4 + c4] - Mt);     // 0 for a group that saw nothing
        const float4 x = s_a[g * v4 + c4];
        r.x += f * x.x; r.y += f * x.y; r.z += f * x.z; r.w += f * x.w;
        lt += f * s_l[g * v4 + c4];
      }
    if (lt > 0.f) {
      const float inv = 1.0f / lt;
      r.x *= inv; r.y *= inv; r.z *= inv; r.w *= inv;
    }
    reinterpret_cast<float4*>(p.o + (size_t)row * p.v)[c4] = r;
  }
}

// Scheduling aid for ragged batches: a permutation of the KV groups by decreasing length
// (counting sort over 1024 length classes; the order inside a class is arbitrary, which only
// affects which workgroup runs when, never a result).  One workgroup.
__global__ __launch_bounds__(1024)
void length_order_kernel(const int32_t* lens, int lens_div, int nseq, int cap, int32_t* order) {
  __shared__ int count[1024];
  __shared__ int start[1024];
  __shared__ int cmin[16], cmax[16];
  __shared__ int wave_total[16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float per_pos = 1023.0f / (float)cap;
  auto cls_of = [&](int L) {
    L = L < 0 ? 0 : (L > cap ? cap : L);
    return 1023 - min(1023, (int)((float)L * per_pos));      // class 0 holds the longest
  };
  // a thread's first kKeep groups stay in registers (every group, up to 4096 of them): the lengths are
  // read from memory once, all loads in flight together, instead of once per pass
  constexpr int kKeep = 4;
  int mine[kKeep];
#pragma unroll
  for (int u = 0; u < kKeep; ++u) {
    const int i = tid + 1024 * u;
    mine[u] = i < nseq ? cls_of(lens[i / lens_div]) : -1;
  }
  auto cls = [&](int i) {                                  // group i = tid + 1024 u of this thread
    const int u = i >> 10;
    int c = u == 0 ? mine[0] : u == 1 ? mine[1] : u == 2 ? mine[2] : u == 3 ? mine[3] : -1;
    return c >= 0 ? c : cls_of(lens[i / lens_div]);
  };
  count[tid] = 0;
  // all groups in one class (equal lengths, the common case): keep the given order and spare the
  // atomics, which would all hit one counter
  int lo = 1023, hi = 0;
  for (int i = tid; i < nseq; i += 1024) {
    const int c = cls(i);
    lo = min(lo, c);
    hi = max(hi, c);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    lo = min(lo, __shfl_xor(lo, off));
    hi = max(hi, __shfl_xor(hi, off));
  }
  if (lane == 0) { cmin[wave] = lo; cmax[wave] = hi; }
  __syncthreads();
  for (int w = 0; w < 16; ++w) { lo = min(lo, cmin[w]); hi = max(hi, cmax[w]); }
  if (lo >= hi) {
    for (int i = tid; i < nseq; i += 1024) order[i] = i;
    return;
  }
  for (int i = tid; i < nseq; i += 1024) atomicAdd(&count[cls(i)], 1);
  __syncthreads();
  // exclusive prefix sum over the classes: inside each wave with shuffles, then over the 16 wave totals
  const int x = count[tid];
  int incl = x;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int y = __shfl_up(incl, off);
    if (lane >= off) incl += y;
  }
  if (lane == 63) wave_total[wave] = incl;
  __syncthreads();
  int before = 0;                                  // classes in earlier waves
  for (int w = 0; w < wave; ++w) before += wave_total[w];
  start[tid] = before + incl - x;
  __syncthreads();
  for (int i = tid; i < nseq; i += 1024) order[atomicAdd(&start[cls(i)], 1)] = i;
}

// Beam search bookkeeping: hypothesis slot r continues hypothesis parent[r], so its cache
// becomes a copy of that hypothesis' valid rows.  One workgroup per (slot, KV head, 64 KiB piece
// of the rows); source and destination are different buffers, so slots may be duplicated or
// dropped freely.  Rows at and beyond the length are not touched.
__global__ __launch_bounds__(256)
void reorder_kernel(const uint4* K_src, const uint4* V_src, const int32_t* lens_src, const int32_t* parent,
                    uint4* K_dst, uint4* V_dst, int32_t* lens_dst, int n, int h_kv, int cap,
                    int k_row16, int v_row16) {
  const int r = blockIdx.x / h_kv, j = blockIdx.x % h_kv;
  int par = parent[r];
  par = par < 0 ? 0 : (par >= n ? n - 1 : par);
  int L = lens_src[par];
  L = L < 0 ? 0 : (L > cap ? cap : L);
  if (blockIdx.y == 0 && j == 0 && threadIdx.x == 0) lens_dst[r] = L;
  const size_t piece = 4096;                       // 16-byte words per workgroup and tensor
  const size_t from = (size_t)blockIdx.y * piece;
  {
    const size_t words = (size_t)L * k_row16;
    const uint4* src = K_src + ((size_t)par * h_kv + j) * cap * k_row16;
    uint4* dst = K_dst + ((size_t)r * h_kv + j) * cap * k_row16;
    const size_t to = min(from + piece, words);
    for (size_t i = from + threadIdx.x; i < to; i += 256) dst[i] = src[i];
  }
  {
    const size_t words = (size_t)L * v_row16;
    const uint4* src = V_src + ((size_t)par * h_kv + j) * cap * v_row16;
    uint4* dst = V_dst + ((size_t)r * h_kv + j) * cap * v_row16;
    const size_t to = min(from + piece, words);
    for (size_t i = from + threadIdx.x; i < to; i += 256) dst[i] = src[i];
  }
}

// In-place form of the listings' concat (Section 2.4 / Section 3): row lens[i]
// of every KV group of sequence i receives the new key / value row, then
// lens[i] grows by one.  One workgroup per sequence, so the length is read by
// all threads before thread 0 updates it.
template <typename T> __device__ __forceinline__ T to_cache(float x);
template <> __device__ __forceinline__ float to_cache<float>(float x) { return x; }
template <> __device__ __forceinline__ uint16_t to_cache<uint16_t>(float x) { return (uint16_t)float_to_bf16_rne(x); }

// n rows per sequence at once (n = 1: one decode step; n > 1: a prompt).  New rows are
// k_new [b, n, h_kv, k]; a sequence that cannot hold all n rows is left untouched.
template <typename T>
__global__ __launch_bounds__(256)
void append_kernel(T* K, T* V, const float* k_new, const float* v_new, int32_t* lens,
                   int h_kv, int cap, int k, int v, int n) {
  const int i = blockIdx.x;
  const int L = lens[i];
  __syncthreads();
  if (L < 0 || L + n > cap) return;
  for (int idx = threadIdx.x; idx < n * h_kv * k; idx += 256) {
    const int r = idx / (h_kv * k), rem = idx - r * (h_kv * k);
    const int j = rem / k, c = rem - j * k;
    K[(((size_t)i * h_kv + j) * cap + L + r) * k + c] = to_cache<T>(k_new[(size_t)i * n * h_kv * k + idx]);
  }
  for (int idx = threadIdx.x; idx < n * h_kv * v; idx += 256) {
    const int r = idx / (h_kv * v), rem = idx - r * (h_kv * v);
    const int j = rem / v, c = rem - j * v;
    V[(((size_t)i * h_kv + j) * cap + L + r) * v + c] = to_cache<T>(v_new[(size_t)i * n * h_kv * v + idx]);
  }
  if (threadIdx.x == 0) lens[i] = L + n;
}

// Streaming read: every 16-byte word is loaded once (non-temporal, as the decode kernel reads
// the cache), folded into a checksum so the loads cannot be dropped.  A wave reads 16 KiB
// contiguous chunks (16 loads of 1 KiB in flight), the granularity of the decode kernel's tiles.
typedef __attribute__((ext_vector_type(4))) uint32_t word16;
__global__ __launch_bounds__(256)
void stream_read_kernel(const word16* src, size_t n16, float* sink) {
  const size_t nwaves = (size_t)gridDim.x * 4;
  const size_t wave = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  uint32_t acc = 0;
  const size_t nchunks = n16 >> 10;                       // 1024 words = 16 KiB
  for (size_t c = wave; c < nchunks; c += nwaves) {
    const word16* base = src + (c << 10) + lane;
    word16 w[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) w[u] = __builtin_nontemporal_load(base + 64 * u);
#pragma unroll
    for (int u = 0; u < 16; ++u) acc ^= w[u].x ^ w[u].y ^ w[u].z ^ w[u].w;
  }
  for (size_t i = (nchunks << 10) + wave * 64 + lane; i < n16; i += nwaves * 64) {      // the last partial chunk
    const word16 a = __builtin_nontemporal_load(src + i);
    acc ^= a.x ^ a.y ^ a.z ^ a.w;
  }
  if (acc == 0x9e3779b9u) sink[blockIdx.x & 4095] = 1.f;   // practically never; keeps the loads live
}

__global__ __launch_bounds__(256)
void stream_copy_kernel(const uint4* src, uint4* dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace

hipError_t launch_combine(const CombineParams& p, hipStream_t st) {
  const size_t total = (size_t)p.rows * (p.v >> 2);
  const dim3 grid((unsigned)((total + 255) / 256)), block(256);
  if (p.PS <= 4) hipLaunchKernelGGL(combine_kernel<4>, grid, block, 0, st, p);
  else if (p.PS <= 16 || p.rows > (1 << 20)) hipLaunchKernelGGL(combine_kernel<8>, grid, block, 0, st, p);
  else hipLaunchKernelGGL(combine_wide_kernel, dim3((unsigned)p.rows), block, 0, st, p);
  return hipGetLastError();
}

hipError_t launch_length_order(const int32_t* lens, int lens_div, int nseq, int cap, int32_t* order, hipStream_t st) {
  hipLaunchKernelGGL(length_order_kernel, dim3(1), dim3(1024), 0, st, lens, lens_div, nseq, cap, order);
  return hipGetLastError();
}

hipError_t launch_reorder(const void* K_src, const void* V_src, const int32_t* lens_src, const int32_t* parent,
                          void* K_dst, void* V_dst, int32_t* lens_dst, int n, int h_kv, int cap,
                          size_t k_row_bytes, size_t v_row_bytes, hipStream_t st) {
  const size_t row16 = (k_row_bytes > v_row_bytes ? k_row_bytes : v_row_bytes) / 16;
  const size_t pieces = ((size_t)cap * row16 + 4095) / 4096;
  const dim3 grid((unsigned)((size_t)n * h_kv), (unsigned)pieces), block(256);
  hipLaunchKernelGGL(reorder_kernel, grid, block, 0, st, (const uint4*)K_src, (const uint4*)V_src, lens_src, parent,
                     (uint4*)K_dst, (uint4*)V_dst, lens_dst, n, h_kv, cap, (int)(k_row_bytes / 16), (int)(v_row_bytes / 16));
  return hipGetLastError();
}

hipError_t launch_append(void* K, void* V, const float* k_new, const float* v_new, int32_t* lens,
                         int b, int h_kv, int cap, int k, int v, int n, int is_bf16, hipStream_t st) {
  if (is_bf16)
    hipLaunchKernelGGL(append_kernel<uint16_t>, dim3(b), dim3(256), 0, st, (uint16_t*)K, (uint16_t*)V,
                       k_new, v_new, lens, h_kv, cap, k, v, n);
  else
    hipLaunchKernelGGL(append_kernel<float>, dim3(b), dim3(256), 0, st, (float*)K, (float*)V,
                       k_new, v_new, lens, h_kv, cap, k, v, n);
  return hipGetLastError();
}

hipError_t launch_stream_read(const void* src, size_t bytes, float* sink, hipStream_t st) {
  hipLaunchKernelGGL(stream_read_kernel, dim3(256), dim3(256), 0, st, (const word16*)src, bytes / 16, sink);
  return hipGetLastError();
}

hipError_t launch_stream_copy(const void* src, void* dst, size_t bytes, hipStream_t st) {
  hipLaunchKernelGGL(stream_copy_kernel, dim3(256 * 16), dim3(256), 0, st, (const uint4*)src, (uint4*)dst, bytes / 16);
  return hipGetLastError();
}

}  // namespace mqa
